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


def _check(mesh, a, b, elem, modes=MODES, seed=0, options=None):
    t1, t2 = O.parse_type(a), O.parse_type(b)
    G = S.random_bytes_array(O.globaltype(t1), elem, seed)
    gview = G.reshape(G.shape[:-1] + (elem,))
    src = [s.reshape(-1).copy() for s in O.distribute(gview.view(np.dtype((np.void, elem)))[..., 0], mesh, t1)]
    src = [np.frombuffer(s.tobytes(), dtype=np.uint8) for s in src]
    want = [np.frombuffer(s.tobytes(), dtype=np.uint8)
            for s in O.distribute(gview.view(np.dtype((np.void, elem)))[..., 0], mesh, t2)]
    for mode in modes:
        plan = R.redist_plan(mesh, a, b, elem, mode, options=options)
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


def test_rank_eight_arrays():
    """The largest rank the boundary accepts: every dim either tiled, moved or untouched, all modes."""
    mesh = {"a": 2, "b": 2, "c": 2}
    _check(mesh, "[2, 2, 1{a}2, 2, 2, 2, 1{b}2, 2]", "[1{c}2, 2, 2, 2, 1{a}2, 2, 2, 1{b}2]", 4, seed=51)
    _check(mesh, "[3, 2{a}4, 2, 5, 1{c}2, 3, 2, 6]", "[3, 4, 1{b}2, 5, 2, 3, 1{a}2, 3{c}6]", 2, seed=52)


def test_tile_shapes_for_runs_that_do_not_fill_a_workgroup():
    """Runs that are no multiple of 256 vectors: rows cut into more column blocks than necessary where that keeps
    80 % of the lanes busy, whole rows with more vectors per thread where those keep clearly more."""
    mesh = {"a": 2, "b": 2, "c": 2}
    # 45*48 four-byte elements = 540 vectors: 7 column blocks of 80 (78 rounded up to whole 128-byte lines), three
    # rows per 256-lane tile
    a, b = "[2{c}4, 36, 45{a,b}180, 48]", "[2{a}4, 18{b}36, 90{c}180, 48]"
    info = R.redist_plan(mesh, a, b, 4, R.MODE_FUSED).op(0)[0]
    assert (info.vec_bytes, info.unroll, info.tc, info.tr) == (16, 1, 80, 3)
    _check(mesh, a, b, 4, modes=[R.MODE_FUSED], seed=5)
    # 8*74 four-byte elements = 148 vectors: five column blocks of 32, eight rows per tile (93 % of the lanes; whole
    # rows, three per tile of 512 vectors, would keep 87 %)
    a, b = "[2{a}4, 2{b}4, 32{c}64, 74]", "[4, 4, 8{c,a,b}64, 74]"
    info = R.redist_plan(mesh, a, b, 4, R.MODE_FUSED).op(0)[0]
    assert (info.vec_bytes, info.unroll, info.tc, info.tr) == (16, 1, 32, 8)
    _check(mesh, a, b, 4, modes=[R.MODE_FUSED], seed=6)
    # 18*74 four-byte elements = 333 vectors: whole rows, three per tile of 1024 vectors (98 % of the lanes against 93 %
    # in seven column blocks of 48)
    a, b = "[4{a}8, 6, 18{c,b}72, 74]", "[4{c}8, 3{a}6, 36{b}72, 74]"
    info = R.redist_plan(mesh, a, b, 4, R.MODE_FUSED).op(0)[0]
    assert (info.vec_bytes, info.unroll, info.tc, info.tr) == (16, 4, 333, 3)
    _check(mesh, a, b, 4, modes=[R.MODE_FUSED], seed=7)


def test_destination_major_order_forced_on_small_odd_problems():
    """The option dest_major_min_bytes = 0 makes every op with replicated boxes destination-major, which puts
    its index arithmetic (partial chunks, ragged tiles, non-uniform boxes, every vector width) under the host model."""
    forced = R.Options(dest_major_min_bytes=0)
    rng = random.Random(123)
    meshes = [{"a": 2, "b": 3}, {"a": 4, "b": 2}, {"a": 2, "b": 2, "c": 2}, {"a": 6}, {"a": 3, "b": 5}]
    shapes = [(12, 30), (60, 6, 4), (30, 1, 12), (120,), (6, 10, 2, 6)]
    seen = 0
    for n in range(60):
        mesh, g = rng.choice(meshes), rng.choice(shapes)
        a, b = _random_type(rng, mesh, g), _random_type(rng, mesh, g)
        elem = rng.choice([1, 2, 4, 8, 16])
        _check(mesh, a, b, elem, seed=n, options=forced)
        plan = R.redist_plan(mesh, a, b, elem, R.MODE_FUSED, options=forced)
        seen += plan.op(0)[0].dest_major
        assert R.redist_plan(mesh, a, b, elem, R.MODE_FUSED).op(0)[0].dest_major == 0   # too small by default
    assert seen >= 15


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


def test_row_complete_descriptors_for_last_dim_steps():
    """Steps that split or merge the last dimension get LDS-staged (row-complete) descriptors; the host
    model checks them for bounds, exactly-once writes, staging-area indexing and against the generic ones."""
    from kernel_model import run_plan as model
    mesh = {"p": 8, "q": 8}
    g = (16, 8, 16, 128)
    cases = [
        ("[16, 8, 16, 16{q}128]", "[16, 8, 16, 128]"),                  # allgather on the last dim
        ("[16, 8, 16, 128]", "[16, 8, 16, 16{p}128]"),                  # dynslice on the last dim
        ("[2{p}16, 8, 16, 128]", "[16, 8, 16, 16{p}128]"),              # alltoall into the last dim
        ("[16, 8, 16, 16{p}128]", "[16, 1{p}8, 16, 128]"),              # alltoall out of the last dim
        ("[2{p}16, 1{q}8, 16, 128]", "[16, 8, 16, 2{p,q}128]"),         # two-element runs
        ("[16, 8, 16, 2{q,p}128]", "[2{q}16, 8, 2{p}16, 128]"),
        ("[16, 8, 2{q}16, 16{p}128]", "[16, 8, 2{p}16, 128]"),          # permute + gather
        ("[16, 8, 16, 16{q}128]", "[16, 8, 16, 2{p,q}128]"),            # slice an already tiled last dim
    ]
    total = 0
    for n, (a, b) in enumerate(cases):
        for elem, modes in ((2, [R.MODE_STEPWISE, R.MODE_FUSED]), (1, [R.MODE_FUSED]), (4, [R.MODE_STEPWISE])):
            t1, t2 = O.parse_type(a), O.parse_type(b)
            G = S.random_bytes_array(g, elem, 700 + n)
            gv = G.view(np.dtype((np.void, elem)))[..., 0]
            src = [np.frombuffer(s.tobytes(), dtype=np.uint8) for s in O.distribute(gv, mesh, t1)]
            want = [s.tobytes() for s in O.distribute(gv, mesh, t2)]
            for mode in modes:
                plan = R.redist_plan(mesh, a, b, elem, mode, options=R.Options(cell_form=0))   # the row-staged kernels
                stats = {}
                got = model(plan, src, stats)
                assert [x.tobytes() for x in got] == want, (a, b, elem, mode)
                total += stats.get("row_ops", 0)
                if elem == 2 and mode == R.MODE_FUSED:
                    assert stats.get("row_ops", 0) == 1 and "lds" in plan.step_kernel(0), (a, b)
    assert total >= 20


def test_row_complete_tiles_of_very_short_rows_hold_up_to_1024_rows():
    """Wide rows of 16 and 32 bytes: a tile is 16 KiB all the same (1024 / 512 rows), ragged at the end of a box."""
    mesh = {"x": 4}
    for a, b, elem, w_log2, r_log2 in [("[2500, 2{x}8]", "[625{x}2500, 8]", 2, 4, 10),     # 4-byte pieces of 16-byte rows
                                      ("[625{x}2500, 4]", "[2500, 1{x}4]", 4, 4, 10),     # scatter of the same
                                      ("[1300, 2{x}8]", "[325{x}1300, 8]", 4, 5, 9)]:     # 8-byte pieces of 32-byte rows
        info = R.redist_plan(mesh, a, b, elem, R.MODE_FUSED).row_op(0)[0]
        assert info.enabled == 1 and info.general == 0 and (info.w_log2, info.r_log2) == (w_log2, r_log2), (a, b)
        _check(mesh, a, b, elem, seed=41)


def test_row_complete_descriptors_when_the_last_dims_are_untouched():
    """A step on the dim in front of untouched last dims moves pieces of (its tile extent) x (their extents): the
    tables are folded so that the staged kernels see those pieces as rows -- also when the untouched dims are
    tiled, the same way on both sides, by the same or by another mesh axis."""
    mesh = {"a": 2, "b": 2, "c": 2}
    cases = [
        ("[6, 2{b}4, 1{a,c}4, 8]", "[6, 4, 4, 8]", 4),                  # gather: 32-byte pieces of 128-byte rows
        ("[6, 3{c}6, 4, 2, 4]", "[3{b}6, 6, 2{a}4, 2, 4]", 2),            # two untouched dims behind a dynslice
        ("[8, 2{b}4, 10{a}20]", "[4{b}8, 4, 10{a}20]", 4),                # untouched last dim tiled by the same axis
        ("[8, 2{b}4, 10{a}20]", "[4{b}8, 4, 10{c}20]", 4),                # ... by another axis: a permute, no last-dim step
        ("[12, 6, 1{a,b}4, 3]", "[6{c}12, 3{a}6, 4, 3]", 4),              # 12-byte pieces: granules off the vector grid
    ]
    staged = 0
    for a, b, elem in cases:
        _check(mesh, a, b, elem, seed=31)
        plan = R.redist_plan(mesh, a, b, elem, R.MODE_FUSED)
        staged += plan.row_op(0)[0].enabled
    assert staged >= 4
    info = R.redist_plan(mesh, cases[0][0], cases[0][1], 4, R.MODE_FUSED).row_op(0)[0]
    assert info.enabled == 1 and info.dir == 0 and (1 << info.w_log2, 1 << info.n_log2, info.n_pieces) == (128, 32, 4)


def test_row_complete_not_used_when_runs_are_long():
    plan = R.redist_plan({"x": 8}, "[64{x}512, 256]", "[512, 32{x}256]", 2, R.MODE_FUSED)        # 64-byte runs, W = 512
    assert plan.row_op(0)[0].enabled == 1
    plan = R.redist_plan({"x": 8}, "[64{x}512, 512]", "[512, 64{x}512]", 2, R.MODE_FUSED)        # 128-byte runs: generic
    assert plan.row_op(0)[0].enabled == 0
    plan = R.redist_plan({"x": 8}, "[64{x}512, 1024]", "[512, 128{x}1024]", 2, R.MODE_FUSED)     # 256-byte runs: generic
    assert plan.row_op(0)[0].enabled == 0
    plan = R.redist_plan({"x": 4, "y": 2}, "[128{x}512, 1024]", "[512, 256{x}1024]", 1, R.MODE_FUSED)   # ... unless a scatter
    assert plan.row_op(0)[0].enabled == 1 and plan.row_op(0)[0].narrow_count == 2                        # writes them twice
    plan = R.redist_plan({"x": 8}, "[64{x}512, 8192]", "[512, 1024{x}8192]", 2, R.MODE_FUSED)   # 2 KiB runs: generic
    assert plan.row_op(0)[0].enabled == 0 and "lds" not in plan.step_kernel(0)
    plan = R.redist_plan({"x": 8}, "[64{x}512, 16, 24]", "[512, 2{x}16, 24]", 2, R.MODE_FUSED)   # last dim untouched:
    assert plan.row_op(0)[0].enabled == 1 and plan.row_op(0)[0].n_bytes == 96                     # 2 x 24 elements per piece
    plan = R.redist_plan({"x": 8}, "[64{x}512, 16, 256]", "[512, 2{x}16, 256]", 2, R.MODE_FUSED)  # ... of 1 KiB: generic
    assert plan.row_op(0)[0].enabled == 0
    plan = R.redist_plan({"x": 4}, "[8{x}32, 96]", "[32, 24{x}96]", 2, R.MODE_FUSED)             # 192-byte rows: general form
    assert plan.row_op(0)[0].enabled == 1 and plan.row_op(0)[0].general == 1


def test_row_complete_general_form_for_sizes_that_are_not_powers_of_two():
    from kernel_model import run_plan as model
    mesh = {"a": 2, "b": 2, "c": 2}
    cases = [
        ((6, 20, 74), "[6, 10{a}20, 74]", "[6, 20, 37{a}74]", 4),               # 148-byte pieces of 296-byte rows
        ((12, 8, 90), "[6{b}12, 8, 90]", "[12, 8, 45{b}90]", 4),
        ((4, 16, 180), "[4, 16, 45{c,b}180]", "[2{c}4, 16, 90{b}180]", 4),
        ((16, 6, 72), "[8{a}16, 6, 72]", "[16, 6, 18{a,c}72]", 4),
        ((8, 24, 24), "[8, 12{a}24, 12{b}24]", "[8, 24, 6{b,a}24]", 8),
        ((10, 12, 156), "[10, 12, 78{b}156]", "[10, 3{b,c}12, 156]", 2),          # gather into 312-byte rows
        ((4, 6, 40), "[4, 6, 5{a,b,c}40]", "[4, 6, 40]", 1),                      # 5-byte pieces, byte vectors
        ((2, 4, 2560), "[2, 4, 320{a,b,c}2560]", "[1{a}2, 4, 2560]", 4),          # W = 10 KiB: too wide, generic body
    ]
    seen_general = 0
    for n, (g, a, b, elem) in enumerate(cases):
        t1, t2 = O.parse_type(a), O.parse_type(b)
        G = S.random_bytes_array(g, elem, 900 + n)
        gv = G.view(np.dtype((np.void, elem)))[..., 0]
        src = [np.frombuffer(s.tobytes(), dtype=np.uint8) for s in O.distribute(gv, mesh, t1)]
        want = [s.tobytes() for s in O.distribute(gv, mesh, t2)]
        for mode in (R.MODE_STEPWISE, R.MODE_FUSED):
            plan = R.redist_plan(mesh, a, b, elem, mode)
            stats = {}
            got = model(plan, src, stats)
            assert [x.tobytes() for x in got] == want, (a, b, elem, mode)
            seen_general += stats.get("general_row_ops", 0)
    assert seen_general >= 10


M3 = {"a": 2, "b": 2, "c": 2}
M1 = {"a": 2}
# (mesh, global shape, source type, destination type, element bytes, granule of the span form; 16 = whole vectors fit,
# no span form needed).  Scatters whose pieces go to several shards keep the row-by-row form.
SPAN_CASES = [
    (M3, (6, 80, 90), "[6, 80, 45{a}90]", "[6, 40{a}80, 90]", 4, 4),             # 180-byte pieces, chunks shorter than a tile, 4 replicas
    (M1, (3, 100, 90), "[3, 50{a}100, 90]", "[3, 100, 45{a}90]", 4, 4),           # scatter, chunks longer than a tile
    (M3, (3, 100, 90), "[3, 50{b}100, 90]", "[3, 100, 45{b}90]", 4, 4),           # scatter to 4 replicas: row-by-row form
    (M1, (2, 64, 74), "[2, 64, 74]", "[2, 64, 37{a}74]", 4, 4),                    # dynslice
    (M3, (4, 24, 296), "[4, 24, 148{a}296]", "[4, 12{a}24, 296]", 4, 16),         # 592-byte pieces: whole vectors
    (M3, (4, 24, 298), "[4, 24, 149{a}298]", "[4, 12{a}24, 298]", 4, 4),          # 596-byte pieces
    (M3, (5, 96, 46), "[5, 96, 23{b}46]", "[5, 48{b}96, 46]", 4, 4),
    (M3, (5, 48, 92), "[5, 48, 46{b}92]", "[5, 24{b}48, 92]", 4, 8),              # 8-byte granules
    (M3, (2, 96, 90), "[2, 96, 45{c}90]", "[2, 48{c}96, 90]", 2, 2),              # bf16, odd element count
    (M1, (2, 96, 90), "[2, 48{a}96, 90]", "[2, 96, 45{a}90]", 2, 2),              # ... scattered
    (M3, (2, 1024, 10), "[2, 1024, 5{c}10]", "[2, 1024, 10]", 1, 1),              # allgather of 5-byte pieces to all shards
    (M1, (2, 2048, 14), "[2, 2048, 14]", "[2, 2048, 7{a}14]", 1, 1),              # 7-byte pieces, byte granules
    (M3, (2, 8, 32, 90), "[2, 8, 32, 45{a}90]", "[1{a}2, 8, 32, 90]", 4, 4),       # outer dims merge into one chunk
    (M3, (2, 8, 64, 90), "[2, 4{b}8, 64, 45{a}90]", "[2, 8, 32{a}64, 90]", 4, 4),
    (M3, (4, 6, 8, 90), "[4, 6, 8, 45{a}90]", "[4, 6, 4{a}8, 90]", 4, 4),           # chunks of 4 rows: several chunks per tile
    (M3, (64, 2, 90), "[64, 1{a}2, 45{b}90]", "[32{b}64, 2, 90]", 4, 4),           # rows not contiguous: every row a chunk
    (M1, (37, 3, 5, 74), "[37, 3, 5, 74]", "[37, 3, 5, 37{a}74]", 2, 2),           # ragged last tile of several chunks
    (M3, (2, 3, 600, 90), "[2, 3, 600, 45{c}90]", "[2, 3, 300{c}600, 90]", 4, 4),   # long chunks cut into stretches, one per tile
    (M3, (4, 16, 10), "[4, 16, 5{a}10]", "[4, 8{a}16, 10]", 2, 2),                 # 10-byte pieces, 64 chunks per tile
    (M3, (64, 4, 10), "[64, 4, 5{a}10]", "[64, 2{a}4, 10]", 2, 16),                # chunks of 2 rows of 10-byte pieces: row-by-row form
]


def test_row_complete_span_form_for_rows_that_start_off_the_vector_grid():
    """Rows whose byte length is not a multiple of 16 start at odd multiples of a granule; when consecutive
    rows are contiguous on both sides the span form covers them with aligned 16-byte blocks.  The host
    model checks block/granule coverage, alignment, staging addresses and the bytes moved."""
    from kernel_model import run_plan as model
    seen = 0
    for n, (mesh, g, a, b, elem, gran) in enumerate(SPAN_CASES):
        t1, t2 = O.parse_type(a), O.parse_type(b)
        G = S.random_bytes_array(g, elem, 1200 + n)
        gv = G.view(np.dtype((np.void, elem)))[..., 0]
        src = [np.frombuffer(s.tobytes(), dtype=np.uint8) for s in O.distribute(gv, mesh, t1)]
        want = [s.tobytes() for s in O.distribute(gv, mesh, t2)]
        for mode in (R.MODE_STEPWISE, R.MODE_FUSED):
            plan = R.redist_plan(mesh, a, b, elem, mode, options=R.Options(cell_form=0))   # the row-staged kernels
            stats = {}
            got = model(plan, src, stats)
            assert [x.tobytes() for x in got] == want, (a, b, elem, mode)
            seen += stats.get("span_row_ops", 0)
            if mode == R.MODE_FUSED and plan.row_op(0)[0].enabled:
                ri = plan.row_op(0)[0]
                assert (ri.span == 1) == (gran < 16 and not (ri.dir == 1 and (ri.narrow_count > 1 or (ri.vw, ri.vn) == (16, 8)))), (a, b, ri.span, ri.vn, ri.vw)
                if ri.span:
                    assert ri.gran == gran and "lds" in plan.step_kernel(0)
    assert seen >= 12


def test_runs_of_dynslices_and_allgathers_are_one_launch():
    """Stepwise plans carry out a run of consecutive dynslices, or of consecutive allgathers, with one launch built
    from the device tables before the run's first and after its last step (problem P4 of the paper's adversarial table
    is three allgathers), and fold a run of dynslices into the launch of the step (or run of allgathers) that follows
    it: the slice is local, the next collective reads the part it keeps.  The naive baseline keeps one launch per step."""
    from kernel_model import run_plan as model
    mesh = {"a": 2, "b": 2, "c": 2}
    cases = [((4, 2, 2, 4, 2, 4), "[2{c}4, 2, 2, 2{a}4, 2, 2{b}4]", "[4, 2, 2, 4, 2, 4]"),          # P4, shrunk
             ((8, 6, 4), "[8, 6, 4]", "[4{a}8, 3{b}6, 2{c}4]"),                                        # three dynslices
             ((8, 6, 4), "[4{a}8, 6, 4]", "[8, 3{b}6, 2{c}4]"),                            # two dynslices, one allgather
             ((8, 12, 4), "[8, 6{a}12, 4]", "[2{a,b}8, 12, 2{c}4]")]           # dynslice(s) in front of an alltoall
    for n, (g, a, b) in enumerate(cases):
        t1, t2 = O.parse_type(a), O.parse_type(b)
        G = S.random_bytes_array(g, 4, 1500 + n)
        gv = G.view(np.dtype((np.void, 4)))[..., 0]
        src = [np.frombuffer(s.tobytes(), dtype=np.uint8) for s in O.distribute(gv, mesh, t1)]
        want = [s.tobytes() for s in O.distribute(gv, mesh, t2)]
        plan = R.redist_plan(mesh, a, b, 4, R.MODE_STEPWISE)
        kinds = [s["kind"] for s in plan.steps()]
        runs = [k for k, (x, y) in enumerate(zip([None] + kinds, kinds)) if not (x == y and x in ("dynslice", "allgather"))]
        if kinds[0] == "dynslice" and len(runs) > 1:
            del runs[1]                                   # the run after the leading dynslices shares their launch
        lasts = [k - 1 for k in runs[1:]] + [len(kinds) - 1]
        assert [plan.op_last_step(k) for k in range(plan.num_ops)] == lasts and plan.num_ops < len(kinds), (a, b, kinds)
        assert plan.step_kernel(0).startswith("redist_" + kinds[lasts[0]])
        assert [x.tobytes() for x in model(plan, src)] == want
        naive = R.redist_plan(mesh, a, b, 4, R.MODE_NAIVE)
        assert naive.num_ops == len(naive.steps())
        assert [x.tobytes() for x in model(naive, src)] == want


def odd_shape_problems(count, seed=77):
    """Seeded random problems on arrays whose last dims are odd multiples of small element counts and whose outer
    dims are large enough for several tiles: the shapes that exercise the staged kernels' general and span forms
    (several chunks per tile, long chunks cut into stretches, ragged last tiles, every granule size)."""
    import random
    from test_planner import _random_type
    rng = random.Random(seed)
    meshes = [{"a": 2, "b": 2, "c": 2}, {"a": 4, "b": 2}, {"a": 2, "b": 3}, {"a": 2}, {"a": 8}]
    shapes = [(96, 40, 90), (50, 12, 74), (6, 300, 46), (2400, 30), (4, 6, 80, 36), (120, 24, 6), (16, 250, 90), (48, 8, 8, 148)]
    out = []
    while len(out) < count:
        mesh, g = rng.choice(meshes), rng.choice(shapes)
        a, b = _random_type(rng, mesh, g), _random_type(rng, mesh, g)
        ta, tb = O.parse_type(a), O.parse_type(b)
        if a == b or ta[-1].c == tb[-1].c:      # keep the problems that split or merge the last dimension
            continue
        out.append((mesh, g, a, b, rng.choice([1, 2, 4, 4, 8])))
    return out


def test_random_odd_shapes_under_the_host_model():
    from kernel_model import run_plan as model
    stats = {}
    for n, (mesh, g, a, b, elem) in enumerate(odd_shape_problems(14)):
        t1, t2 = O.parse_type(a), O.parse_type(b)
        G = S.random_bytes_array(g, elem, 1700 + n)
        gv = G.view(np.dtype((np.void, elem)))[..., 0]
        src = [np.frombuffer(s.tobytes(), dtype=np.uint8) for s in O.distribute(gv, mesh, t1)]
        want = [s.tobytes() for s in O.distribute(gv, mesh, t2)]
        for mode in (R.MODE_STEPWISE, R.MODE_FUSED):
            got = model(R.redist_plan(mesh, a, b, elem, mode), src, stats)
            assert [x.tobytes() for x in got] == want, (mesh, a, b, elem, mode)
    assert stats.get("span_row_ops", 0) >= 4 and stats.get("general_row_ops", 0) > stats.get("span_row_ops", 0), stats


def test_destination_major_order_with_several_chunks():
    """Ops of 32 MiB and more whose boxes all go to the same number of shards are taken chunk by chunk (16 MiB of
    source), destination by destination within a chunk, chunks running across boxes: two shards of 40.6 MiB give
    five whole chunks and a partial one.  Smaller ops are stored to their destinations in turn."""
    from kernel_model import run_plan as model
    mesh = {"x": 2}
    g, a, b, elem = (2 * 2600, 1024), "[2600{x}5200, 1024]", "[5200, 1024]", 16
    t1, t2 = O.parse_type(a), O.parse_type(b)
    G = S.random_bytes_array(g, elem, 1900)
    gv = G.view(np.dtype((np.void, elem)))[..., 0]
    src = [np.frombuffer(s.tobytes(), dtype=np.uint8) for s in O.distribute(gv, mesh, t1)]
    want = [s.tobytes() for s in O.distribute(gv, mesh, t2)]
    plan = R.redist_plan(mesh, a, b, elem, R.MODE_STEPWISE, options=R.Options(dest_major_fanout=1))
    info, boxes, _ = plan.op(0)
    assert info.dest_major == 1 and info.unroll == 1 and info.chunk_tiles == 4096
    assert info.dm_count == 2 and info.src_tiles == 20800 and info.n_tiles == 41600
    # by default a workgroup stores to both shards: one group, as many workgroups as tiles
    dflt = R.redist_plan(mesh, a, b, elem, R.MODE_STEPWISE).op(0)[0]
    assert (dflt.dest_major, dflt.dm_fanout, dflt.dm_groups, dflt.n_tiles) == (1, 2, 1, 20800)
    assert all(bx.dst_count == 2 and bx.n_tiles == 10400 for bx in boxes)
    assert [x.tobytes() for x in model(plan, src)] == want
    small = R.redist_plan(mesh, "[64{x}128, 1024]", "[128, 1024]", elem, R.MODE_STEPWISE)
    info, boxes, _ = small.op(0)
    assert info.dest_major == 0 and info.dm_count == 1 and info.n_tiles == info.src_tiles
    assert all(bx.dst_count == 2 for bx in boxes)


def test_destination_major_order_reads_whole_shards_front_to_back():
    """For this order every box reads the lowest-numbered holder of its tile, boxes are cut into pieces that are
    contiguous in the source, and the pieces are sorted by source address: chunks are dense stretches of memory
    (pieces lying a power of two apart would share cache sets), and together the pieces tile every shard read."""
    from kernel_model import run_plan as model
    mesh, elem = {"p": 2, "q": 2}, 16
    cases = [
        # source tiled over both axes, target replicated over p: whole 16 MiB shards, two 8 MiB boxes each
        ((4, 4, 128, 2048), "[4, 2{p}4, 64{q}128, 2048]", "[2{q}4, 4, 128, 2048]", 8, 4),
        # replicated source, target tiled over q: boxes of 8 rows of 4 MiB lying 8 MiB apart are cut into rows,
        # all read from shard 0, which they tile once sorted
        ((8, 4, 128, 1024), "[8, 4, 128, 1024]", "[8, 2{q}4, 128, 1024]", 16, 1),
    ]
    for g, a, b, n_boxes, n_src in cases:
        t1, t2 = O.parse_type(a), O.parse_type(b)
        # (one destination per workgroup: two groups, so every chunk is read twice and the source order applies)
        plan = R.redist_plan(mesh, a, b, elem, R.MODE_FUSED, options=R.Options(dest_major_fanout=1))
        info, boxes, _ = plan.op(0)
        assert info.dest_major == 1 and info.dm_count == 2 and info.dm_groups == 2 and len(boxes) == n_boxes, (a, b, len(boxes))
        assert len({bx.src_dev for bx in boxes}) == n_src
        at = {}
        for bx in boxes:                                    # source order, gap-free within a shard
            assert bx.src_off == at.get(bx.src_dev, 0), (a, b)
            at[bx.src_dev] = bx.src_off + bx.rows * bx.run_vecs * info.vec_bytes
        assert all(v == info.src_shard_bytes for v in at.values())
        assert [bx.src_dev for bx in boxes] == sorted(bx.src_dev for bx in boxes)
        G = S.random_bytes_array(g, elem, 1901)
        gv = G.view(np.dtype((np.void, elem)))[..., 0]
        src = [np.frombuffer(s.tobytes(), dtype=np.uint8) for s in O.distribute(gv, mesh, t1)]
        want = [s.tobytes() for s in O.distribute(gv, mesh, t2)]
        assert [x.tobytes() for x in model(plan, src)] == want
        # by default both destinations share a workgroup: one group, nothing is read twice, and the pieces go in
        # destination order instead
        plan = R.redist_plan(mesh, a, b, elem, R.MODE_FUSED)
        info, boxes, _ = plan.op(0)
        assert info.dest_major == 1 and info.dm_groups == 1 and len(boxes) == n_boxes
        keys = [(bx.dst_first, bx.dst_off) for bx in boxes]
        assert keys == sorted(keys)
        assert [x.tobytes() for x in model(plan, src)] == want


ROW_DM_CASES = [
    # scatter: every 256-byte piece of the 512-byte source rows goes to 2 shards
    ({"p": 2, "q": 2}, (4, 16, 1024, 128), "[2{p}4, 16, 1024, 128]", "[4, 16, 1024, 64{p}128]", 4, 1),
    # gather: 256-byte rows from two 128-byte pieces, written to 2 shards; the sources are replicated too
    ({"p": 2, "q": 2}, (8, 16, 1024, 128), "[8, 16, 1024, 64{p}128]", "[4{q}8, 16, 1024, 128]", 2, 0),
]


# general and span forms in destination-major order (small: forced by the option; full size: by their 32 MiB and more)
ROW_DM_GENERAL_SMALL = [
    ({"a": 2, "b": 2, "c": 2}, (6, 40, 90), "[6, 40, 45{a}90]", "[6, 20{b}40, 90]", 4),     # span gather, 4 receivers
    ({"a": 2, "b": 2, "c": 2}, (6, 40, 90), "[6, 20{b}40, 90]", "[6, 40, 45{a}90]", 4),     # general scatter, 4 receivers
    ({"a": 2, "b": 2, "c": 2}, (4, 24, 48), "[4, 24, 24{a}48]", "[4, 12{b}24, 48]", 2),     # general gather
    ({"a": 2, "b": 2, "c": 2}, (4, 24, 48), "[4, 12{b}24, 48]", "[4, 24, 12{a,c}48]", 4),   # general scatter, 2 receivers
    ({"a": 2, "b": 2, "c": 2}, (8, 30, 74), "[8, 30, 37{c}74]", "[8, 30, 74]", 4),          # span gather to full replicas
]
ROW_DM_GENERAL_FULL = [
    ({"a": 2, "b": 2, "c": 2}, (256, 312, 312), "[256, 78{c,b}312, 156{a}312]", "[256, 312, 78{c,b}312]", 4, (1, 0)),
    ({"a": 2, "b": 2, "c": 2}, (8, 368, 74, 4, 74), "[8, 368, 37{c}74, 2{a}4, 37{b}74]", "[8, 368, 74, 4, 74]", 4, (1, 1)),
    ({"a": 2, "b": 2, "c": 2}, (741, 96, 160), "[741, 48{c}96, 80{a}160]", "[741, 96, 40{a,b}160]", 4, (1, 0)),
]
# row-by-row general form with 4-byte vectors: instruction-bound, keeps the usual order
ROW_DM_GENERAL_EXCLUDED = ({"a": 2, "b": 2, "c": 2}, "[1024{c}2048, 78{a}156, 74]", "[2048, 156, 37{b}74]", 4)


def test_destination_major_order_of_the_general_and_span_forms():
    forced = R.Options(dest_major_min_bytes=0)
    kinds = set()
    for n, (mesh, g, a, b, elem) in enumerate(ROW_DM_GENERAL_SMALL):
        plan = _check(mesh, a, b, elem, modes=[R.MODE_FUSED], seed=60 + n, options=forced)
        ri = plan.row_op(0)[0]
        assert ri.enabled == 1 and ri.general == 1 and ri.dest_major == 1 and ri.dm_count > 1, (a, b)
        assert ri.n_tiles == ri.src_tiles * ri.dm_groups and ri.dm_groups == -(-ri.dm_count // ri.dm_fanout)
        kinds.add((ri.span, ri.dir))
        assert R.redist_plan(mesh, a, b, elem, R.MODE_FUSED).row_op(0)[0].dest_major == 0       # too small by default
    assert {(1, 0), (0, 1), (0, 0)} <= kinds
    for mesh, g, a, b, elem, (general, span) in ROW_DM_GENERAL_FULL:                             # descriptors only
        ri = R.redist_plan(mesh, a, b, elem, R.MODE_FUSED).row_op(0)[0]
        assert (ri.enabled, ri.general, ri.span, ri.dest_major) == (1, general, span, 1) and ri.chunk_tiles == 1024, (a, b)
    mesh, a, b, elem = ROW_DM_GENERAL_EXCLUDED
    ri = R.redist_plan(mesh, a, b, elem, R.MODE_FUSED).row_op(0)[0]
    assert (ri.enabled, ri.general, ri.span, ri.vn, ri.vw, ri.narrow_count, ri.dest_major) == (1, 1, 0, 4, 4, 4, 0)


def test_destination_major_order_of_the_staged_kernels():
    """Staged (power-of-two form) ops of 32 MiB and more that write every tile to m > 1 shards stage a tile once per
    receiving shard, chunk by chunk, boxes in source order, sources the lowest-numbered holders."""
    from kernel_model import run_plan as model
    for mesh, g, a, b, elem, direction in ROW_DM_CASES:
        t1, t2 = O.parse_type(a), O.parse_type(b)
        plan = R.redist_plan(mesh, a, b, elem, R.MODE_FUSED)
        info, boxes, pieces, dev_list = plan.row_op(0)
        assert info.enabled == 1 and info.general == 0 and info.dir == direction, (a, b)
        assert info.dest_major == 1 and info.dm_count == 2 and info.chunk_tiles == 1024
        assert info.src_tiles == 2048 and (info.dm_fanout, info.dm_groups, info.n_tiles) == (2, 1, 2048)
        one = R.redist_plan(mesh, a, b, elem, R.MODE_FUSED, options=R.Options(dest_major_fanout=1)).row_op(0)[0]
        assert (one.dm_fanout, one.dm_groups, one.n_tiles) == (1, 2, 4096)
        G = S.random_bytes_array(g, elem, 1902)
        gv = G.view(np.dtype((np.void, elem)))[..., 0]
        src = [np.frombuffer(s.tobytes(), dtype=np.uint8) for s in O.distribute(gv, mesh, t1)]
        want = [s.tobytes() for s in O.distribute(gv, mesh, t2)]
        assert [x.tobytes() for x in model(plan, src)] == want
    # below 32 MiB: every tile staged once and stored to all its shards in turn
    info = R.redist_plan({"p": 2, "q": 2}, "[2{p}4, 16, 256, 128]", "[4, 16, 256, 64{p}128]", 4, R.MODE_FUSED).row_op(0)[0]
    assert info.enabled == 1 and info.dest_major == 0 and info.dm_count == 1 and info.n_tiles == info.src_tiles



def cell_problems(count, seed=5):
    """Seeded random problems for the cell-staged kernel (forced on with cell_form = 2): small arrays whose inner dims
    are tiled differently on the two sides, and arrays with a long dim in front of them, so that boxes take several
    tiles and end in a ragged one."""
    rng = random.Random(seed)
    meshes = [{"a": 2, "b": 2, "c": 2}, {"a": 4, "b": 2}, {"a": 2, "b": 3}, {"a": 8}, {"a": 2, "b": 2}]
    shapes = [(6, 8, 12, 8), (10, 6, 4, 24), (4, 12, 6, 18), (20, 4, 74), (3, 8, 6, 4, 16), (8, 36, 8), (12, 4, 4, 37),
              (16, 18, 8), (5, 6, 6, 6, 6), (600, 12, 8), (64, 50, 6, 12), (4, 900, 4, 10), (2, 1100, 8, 6)]
    out = []
    while len(out) < count:
        mesh, g = rng.choice(meshes), rng.choice(shapes)
        a, b = _random_type(rng, mesh, g), _random_type(rng, mesh, g)
        if a != b:
            out.append((mesh, g, a, b, rng.choice([1, 2, 4, 4, 4, 8])))
    return out


def test_cell_complete_descriptors_under_the_host_model():
    """Every launch that qualifies runs as a cell-staged one (cell_form = 2); the model walks its descriptors as the
    kernel does -- bounds on both sides and in the staging area, every granule read from staged bytes, every
    destination byte written once -- and the result must equal the oracle's slices."""
    forced = R.Options(cell_form=2)
    seen, multi_tile, ragged = set(), 0, 0
    for n, (mesh, g, a, b, elem) in enumerate(cell_problems(40)):
        plan = _check(mesh, a, b, elem, modes=[R.MODE_STEPWISE, R.MODE_FUSED], seed=n, options=forced)
        for k in range(plan.num_ops):
            ci, boxes, _ = plan.cell_op(k)
            if ci.enabled:
                assert plan.step_kernel(k).endswith("_cell_kernel")
                seen.add((ci.n_cell, ci.gran, ci.vs, ci.vd, ci.rep > 1))
                multi_tile += any(bx.row_tiles > 1 for bx in boxes)
                ragged += any(bx.len[ci.n_outer - 1] % ci.rows_per_tile for bx in boxes)
    assert {c[0] for c in seen} == {1, 2, 3} and {c[1] for c in seen} == {4, 8, 16}, seen
    assert any(c[4] for c in seen) and any(c[2] != c[3] for c in seen), seen
    assert multi_tile >= 3 and ragged >= 3, (multi_tile, ragged)


def test_cell_complete_form_is_chosen_where_stretches_are_short():
    """Default options: the two slowest paper-shaped problems (two shards alternate every 144 and every 48 bytes in
    the destination) run cell-staged with stretches of kilobytes; a plain last-dim step keeps the row-staged kernel."""
    mesh = {"a": 2, "b": 2, "c": 2}
    for a, b, min_stretch in (("[48, 74, 16{b}32, 9{a,c}36, 8]", "[48, 74, 32, 18{a}36, 4{b}8]", 4096),
                              ("[360, 45{b}90, 36, 1{c,a}4, 24]", "[360, 90, 18{c}36, 2{a}4, 12{b}24]", 3456)):
        plan = R.redist_plan(mesh, a, b, 4, R.MODE_FUSED)
        ci = plan.cell_op(0)[0]
        assert ci.enabled and ci.n_cell >= 2 and ci.min_stretch >= min_stretch
        assert plan.step_kernel(0) == "redist_fused_gather_cell_kernel"
        assert plan.algorithmic_bytes(R.BYTES_MOVED_BY_PLAN) == ci.bytes_read + ci.bytes_written
        assert not R.redist_plan(mesh, a, b, 4, R.MODE_FUSED, options=R.Options(cell_form=0)).cell_op(0)[0].enabled
    plan = R.redist_plan({"x": 8}, "[512{x}4096, 8192]", "[4096, 1024{x}8192]", 2, R.MODE_FUSED)
    assert not plan.cell_op(0)[0].enabled


SIBLING_CASES = [   # (mesh, global shape, src, dst, elem, pieces per run, destinations)
    ({"a": 2, "b": 2}, (4, 6, 512), "[4, 6, 256{a}512]", "[4, 6, 512]", 4, 2, 4),                 # 1 KiB pieces to 4 replicas
    ({"a": 4, "b": 2}, (3, 10, 2048), "[3, 10, 512{a}2048]", "[3, 5{b}10, 2048]", 4, 4, 4),       # 2 KiB pieces, 4 per row
    ({"a": 2, "b": 2, "c": 2}, (2, 9, 384), "[2, 9, 192{c}384]", "[1{a}2, 9, 384]", 16, 2, 4),    # 3 KiB pieces of 16-byte elements
    ({"a": 2, "b": 3}, (5, 7, 444), "[5, 7, 148{b}444]", "[5, 7, 444]", 4, 3, 6),                 # 592-byte pieces, three per row
    ({"x": 2, "y": 4, "z": 4}, (16, 24, 4096), "[2{x,y}16, 24, 1024{z}4096]", "[16, 24, 4096]", 2, 4, 32),   # the 32-shard gather, reduced
]


def test_sibling_boxes_take_turns_tile_by_tile():
    """Destination-major ops whose destination rows are pieces under 4 KiB from several shards: the sibling boxes
    stand side by side and their tiles alternate, so that workgroups running together fill the same rows.  The model
    follows the kernel (group and sibling of a tile by division, no descriptor needed) and checks bounds and
    exactly-once writes; the option switches the alternation off or limits the pieces' length; pieces under 512 bytes
    are left alone."""
    forced = R.Options(dest_major_min_bytes=0)
    for n, (mesh, g, a, b, elem, pieces, m) in enumerate(SIBLING_CASES):
        for fan in (0, 1, 2):
            o = R.Options(dest_major_min_bytes=0, dest_major_fanout=fan)
            plan = _check(mesh, a, b, elem, modes=[R.MODE_FUSED], seed=70 + n, options=o)
            info, boxes, _ = plan.op(0)
            assert info.dest_major == 1 and info.dm_count == m and info.sib_count == pieces, (a, b, info.sib_count)
            assert info.tiles_per_box > 0 and len(boxes) % pieces == 0
            for q in range(0, len(boxes), pieces):          # a group: one shape, different shards, adjacent runs
                grp = boxes[q:q + pieces]
                assert len({bx.src_dev for bx in grp}) == pieces and len({bx.dst_first for bx in grp}) == 1
                run_bytes = grp[0].run_vecs * info.vec_bytes
                assert [bx.dst_off - grp[0].dst_off for bx in grp] == [k * run_bytes for k in range(pieces)]
        _check(mesh, a, b, elem, modes=[R.MODE_STEPWISE], seed=80 + n, options=forced)
        off = R.redist_plan(mesh, a, b, elem, R.MODE_FUSED, options=R.Options(dest_major_min_bytes=0, sibling_sources=0))
        assert off.op(0)[0].sib_count == 1 and off.op(0)[0].src_tiles == plan.op(0)[0].src_tiles
    mesh = {"a": 2, "b": 2}
    plan = R.redist_plan(mesh, "[4, 6, 64{a}128]", "[4, 6, 128]", 4, R.MODE_FUSED, options=forced)   # 256-byte pieces
    assert plan.op(0)[0].sib_count == 1
    a, b = "[4, 6, 1024{a}2048]", "[4, 6, 2048]"                                                      # 4 KiB pieces
    assert R.redist_plan(mesh, a, b, 4, R.MODE_FUSED, options=forced).op(0)[0].sib_count == 2
    limited = R.Options(dest_major_min_bytes=0, sibling_sources=4096)                                 # (the limit, in bytes)
    assert R.redist_plan(mesh, a, b, 4, R.MODE_FUSED, options=limited).op(0)[0].sib_count == 1


ORDINARY_SIBLING_CASES = [   # (mesh, global shape, src, dst, elem, boxes per group, side whose rows the siblings share)
    ({"x": 8}, (64, 4096), "[8{x}64, 4096]", "[64, 512{x}4096]", 2, 8, "src"),       # rows dealt out in 1 KiB pieces
    ({"x": 8}, (64, 4096), "[64, 512{x}4096]", "[8{x}64, 4096]", 2, 8, "dst"),       # and collected again
    ({"b": 3}, (12, 5, 888), "[4{b}12, 5, 888]", "[12, 5, 296{b}888]", 2, 3, "src"),            # 592-byte pieces, three a row
    ({"a": 16}, (16, 3, 8192), "[1{a}16, 3, 8192]", "[16, 3, 512{a}8192]", 4, 8, "src"),         # chains of 16: groups of 8
    ({"a": 2, "b": 2}, (6, 4, 1024), "[6, 2{b}4, 512{a}1024]", "[3{a}6, 2{b}4, 1024]", 4, 2, "dst"),
]


def test_sibling_boxes_of_ordinary_ops():
    """Ops in the ordinary order alternate the tiles of sibling boxes too: boxes whose runs are adjacent pieces of the
    destination's rows, or (boxes then sorted by source) of the source's rows.  The model maps tiles to boxes as the
    kernel does and checks bounds and exactly-once writes in both modes; the option switches it off, and the box
    order is then the usual one."""
    for n, (mesh, g, a, b, elem, p, side) in enumerate(ORDINARY_SIBLING_CASES):
        plan = _check(mesh, a, b, elem, modes=[R.MODE_FUSED], seed=170 + n, options=R.Options(cell_form=0, lds_staging=0))
        _check(mesh, a, b, elem, modes=[R.MODE_STEPWISE], seed=180 + n)
        info, boxes, _ = plan.op(0)
        assert info.dest_major == 0 and info.sib_count == p and plan.step_kernel(0) == "redist_fused_gather_kernel", (a, b, info.sib_count)
        assert info.tiles_per_box > 0 and len(boxes) % p == 0 and info.unroll == 1 and info.vec_bytes == 16
        for q in range(0, len(boxes), p):
            grp = boxes[q:q + p]
            run_bytes = grp[0].run_vecs * info.vec_bytes
            assert 512 <= run_bytes < 4096
            if side == "src":
                assert len({bx.src_dev for bx in grp}) == 1 and len({bx.dst_first for bx in grp}) == p
                assert [bx.src_off - grp[0].src_off for bx in grp] == [k * run_bytes for k in range(p)]
            else:
                assert len({bx.dst_first for bx in grp}) == 1
                assert [bx.dst_off - grp[0].dst_off for bx in grp] == [k * run_bytes for k in range(p)]
        off = R.redist_plan(mesh, a, b, elem, R.MODE_FUSED, options=R.Options(cell_form=0, lds_staging=0, sibling_sources=0))
        oi, ob, _ = off.op(0)
        assert oi.sib_count == 1 and oi.src_tiles == info.src_tiles
        assert [bx.dst_first for bx in ob] == sorted(bx.dst_first for bx in ob)      # destination after destination


def test_sibling_boxes_with_runs_of_several_tiles():
    """Sibling boxes whose runs are two and four tiles wide: the tiles of a run stay together, the runs alternate.
    Both orders (ordinary and destination-major); pieces of the source's rows and runs of three tiles are left in the
    usual order."""
    wide = R.Options(sibling_sources=65536, cell_form=0, lds_staging=0)
    cases = [({"x": 4}, "[12, 2048{x}8192]", "[3{x}12, 8192]", 4, 4, 1),                 # 8 KiB runs, destination side
             ({"x": 4}, "[3{x}12, 8192]", "[12, 2048{x}8192]", 4, 1, 0),                 # source side: under 4 KiB only
             ({"x": 2, "y": 2}, "[6, 4096{x}8192]", "[3{y}6, 8192]", 4, 2, 2),           # 16 KiB runs, two replicas each
             ({"x": 2}, "[5, 3072{x}6144]", "[5, 6144]", 4, 1, 0)]                        # 12 KiB runs: three tiles
    for n, (mesh, a, b, elem, p, lg) in enumerate(cases):
        o = R.Options(sibling_sources=65536, cell_form=0, lds_staging=0, dest_major_min_bytes=0 if n == 2 else 1 << 40)
        plan = _check(mesh, a, b, elem, modes=[R.MODE_FUSED], seed=190 + n, options=o)
        info = plan.op(0)[0]
        assert (info.sib_count, info.sib_inner_log2, info.tr) == (p, lg, 1), (a, b, info.sib_count, info.sib_inner_log2)
        assert info.dest_major == (1 if n == 2 else 0)
        _check(mesh, a, b, elem, modes=[R.MODE_STEPWISE], seed=195 + n, options=wide)


def test_staged_boxes_are_cut_and_sorted_by_destination_address():
    """Power-of-two staged ops in the usual order: boxes whose tiles would leave gaps in the destination (another
    source shard fills them later) are cut into destination-contiguous parts of whole tiles, sorted by where they
    write; lds_staging=2 keeps the boxes; boxes that are one stretch of the destination already are left alone."""
    mesh = {"q": 2, "p": 2}
    a, b = "[2{q}4, 4, 256{p}512, 128]", "[4, 2{p}4, 512, 64{q}128]"          # seq blocks of two shards per destination row
    plan = _check(mesh, a, b, 1, modes=[R.MODE_FUSED], seed=210, options=R.Options(cell_form=0))
    info, boxes, pieces, dev_list = plan.row_op(0)
    assert info.enabled and info.dir == 1 and not info.general and info.dest_major == 0
    assert (info.w_bytes, info.n_bytes, 1 << info.r_log2, info.tiles_per_box) == (128, 64, 128, 2)
    where = [(dev_list[pieces[bx.piece_first].dev_first], pieces[bx.piece_first].narrow_off) for bx in boxes]
    assert where == sorted(where) and len(set(where)) == len(where)
    assert len({dev_list[bx.wide_first] for bx in boxes[:2]}) == 2               # neighbours come from different shards
    kept = R.redist_plan(mesh, a, b, 1, R.MODE_FUSED, options=R.Options(cell_form=0, lds_staging=2))
    kinfo = kept.row_op(0)[0]
    assert kinfo.n_boxes * 4 == info.n_boxes and kinfo.tiles_per_box == 8 and kinfo.n_tiles == info.n_tiles
    _check(mesh, a, b, 1, modes=[R.MODE_STEPWISE], seed=211)
    a, b = "[2{p}4, 4, 256, 128]", "[4, 4, 128{q}256, 64{p}128]"                 # every box one stretch of its destination
    winfo, kinfo = (R.redist_plan(mesh, a, b, 1, R.MODE_FUSED, options=R.Options(cell_form=0, lds_staging=k)).row_op(0)[0]
                    for k in (1, 2))
    assert winfo.enabled and (winfo.n_boxes, winfo.tiles_per_box) == (kinfo.n_boxes, kinfo.tiles_per_box) == (4, 8)


def test_sibling_boxes_on_a_mesh_of_256_devices():
    """Chains of 256 sibling boxes (rows dealt out in 512-byte pieces to every device, and collected again) alternate
    in groups of 8; bounds and exactly-once writes under the host model."""
    mesh = {"x": 64, "y": 4}
    for n, (a, b) in enumerate((("[1{x,y}256, 8192]", "[256, 32{x,y}8192]"), ("[256, 32{x,y}8192]", "[1{x,y}256, 8192]"))):
        plan = _check(mesh, a, b, 16, modes=[R.MODE_FUSED], seed=220 + n)
        info, boxes, _ = plan.op(0)
        assert info.sib_count == 8 and info.dest_major == 0 and len(boxes) == 256 * 256 and info.tiles_per_box == 1

