"""Thin ctypes binding of libredist.so (the C-ABI declared in include/redist.h).

Argument marshalling only: every step of a redistribution runs in the library's HIP kernels.
PyTorch, when used, only supplies device memory (tensor.data_ptr()) and the current stream.
There is no CPU fallback: a missing library raises at import of the first symbol.
"""
from __future__ import annotations

import ctypes
import os
import re
from ctypes import POINTER, c_char_p, c_int32, c_int64, c_uint32, c_void_p

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libredist.so")

MODE_STEPWISE, MODE_FUSED, MODE_NAIVE, MODE_AUTO = 0, 1, 2, 3
STEP_DYNSLICE, STEP_ALLGATHER, STEP_ALLTOALL, STEP_ALLPERMUTE, STEP_FUSED = 0, 1, 2, 3, 4
STEP_NAMES = {0: "dynslice", 1: "allgather", 2: "alltoall", 3: "allpermute", 4: "fused"}
BYTES_READ_MIN, BYTES_READ_LOGICAL, BYTES_WRITE, BYTES_MOVED_BY_PLAN = 0, 1, 2, 3
MAX_RANK, MAX_DEVICES, MAX_EXEC_DEVICES = 8, 4096, 128
STATIC_SCRATCH_BYTES, STATIC_DESC_BYTES = 32 << 20, 1 << 20


class RedistError(RuntimeError):
    def __init__(self, status, message):
        super().__init__("redist status %d: %s" % (status, message))
        self.status = status


class _Mesh(ctypes.Structure):
    _fields_ = [("n_axes", c_int32), ("axis_size", POINTER(c_int64))]


class Options(ctypes.Structure):
    """redist_options: how a plan is lowered to launches.  Options() holds the library's defaults."""
    _fields_ = [("struct_size", c_uint32), ("merge_runs", c_int32), ("fold_permute", c_int32), ("lds_staging", c_int32),
                ("span_form", c_int32), ("dest_major", c_int32), ("unroll", c_int32),
                ("dest_major_min_bytes", c_int64), ("max_grid", c_uint32), ("reserved", c_uint32),
                ("step_latency_elems", c_int64), ("launch_latency_ns", c_int32), ("sustained_gbs", c_int32),
                ("dest_major_fanout", c_int32), ("sibling_sources", c_int32), ("cell_form", c_int32)]

    def __init__(self, **kw):
        super().__init__()
        lib().redist_options_init(ctypes.byref(self))
        for k, v in kw.items():
            if k not in dict(self._fields_):
                raise TypeError("unknown option %r" % k)
            setattr(self, k, v)


class _Type(ctypes.Structure):
    _fields_ = [("rank", c_int32), ("global_shape", POINTER(c_int64)), ("n_axes_of_dim", POINTER(c_int32)),
                ("axes_flat", POINTER(c_int32))]


class Box(ctypes.Structure):
    _fields_ = [("src_off", c_int64), ("dst_off", c_int64), ("src_dev", c_int32), ("dst_first", c_int32),
                ("dst_count", c_int32), ("run_vecs", c_uint32), ("rows", c_uint32), ("tile_first", c_uint32),
                ("col_blocks", c_uint32), ("n_tiles", c_uint32), ("len", c_uint32 * 7), ("magic", c_uint32 * 7),
                ("shift", ctypes.c_uint8 * 7), ("pad0", ctypes.c_uint8), ("dst_dev0", c_int32), ("cb_magic", c_uint32),
                ("cb_shift", ctypes.c_uint8), ("pad", ctypes.c_uint8 * 7)]


class OpInfo(ctypes.Structure):
    _fields_ = [("kind", c_int32), ("n_boxes", c_int32), ("n_dst_list", c_int32), ("n_outer", c_int32),
                ("vec_bytes", c_int32), ("tc", c_int32), ("tr", c_int32), ("tc_magic", c_uint32), ("tc_shift", c_uint32),
                ("dest_major", c_int32), ("n_tiles", c_uint32), ("tiles_per_box", c_uint32),
                ("unroll", c_int32), ("nontemporal", c_int32), ("tpb_magic", c_uint32), ("tpb_shift", c_uint32),
                ("sstride", c_int64 * 7), ("dstride", c_int64 * 7), ("src_shard_bytes", c_int64),
                ("dst_shard_bytes", c_int64), ("chunk_tiles", c_uint32), ("src_tiles", c_uint32),
                ("dm_count", c_uint32), ("dm_magic", c_uint32), ("dm_shift", c_uint32), ("max_grid", c_uint32),
                ("dm_fanout", c_uint32), ("dm_groups", c_uint32), ("sib_count", c_uint32), ("sib_magic", c_uint32),
                ("sib_shift", c_uint32), ("sib_inner_log2", c_uint32)]


class RowBox(ctypes.Structure):
    _fields_ = [("wide_off", c_int64), ("wide_first", c_int32), ("wide_count", c_int32), ("piece_first", c_int32),
                ("rows", c_uint32), ("tile_first", c_uint32), ("n_tiles", c_uint32), ("len", c_uint32 * 7),
                ("magic", c_uint32 * 7), ("shift", ctypes.c_uint8 * 7), ("tpc_shift", ctypes.c_uint8),
                ("chunk_rows", c_uint32), ("tpc", c_uint32), ("tpc_magic", c_uint32), ("n_vchunks", c_uint32),
                ("vrows", c_uint32), ("pad", ctypes.c_uint8 * 12)]


class Piece(ctypes.Structure):
    _fields_ = [("narrow_off", c_int64), ("dev_first", c_int32), ("pad", c_int32)]


class CellBox(ctypes.Structure):
    _fields_ = [("src_off", c_int64), ("dst_off", c_int64), ("src_first", c_int32), ("dst_first", c_int32),
                ("tile_first", c_uint32), ("n_tiles", c_uint32), ("row_tiles", c_uint32), ("rt_magic", c_uint32),
                ("len", c_uint32 * 7), ("magic", c_uint32 * 7), ("shift", ctypes.c_uint8 * 7),
                ("rt_shift", ctypes.c_uint8), ("pad", ctypes.c_uint8 * 8)]


class CellInfo(ctypes.Structure):
    _fields_ = [("enabled", c_int32), ("n_outer", c_int32), ("n_cell", c_int32), ("ps", c_int32), ("pd", c_int32),
                ("rep", c_int32), ("vs", c_int32), ("vd", c_int32), ("gran", c_int32), ("base_first", c_int32),
                ("rows_per_tile", c_uint32), ("src_row_bytes", c_uint32), ("dst_row_bytes", c_uint32),
                ("part_pitch", c_uint32), ("drow_gran", c_uint32), ("dext", c_uint32 * 3), ("piece", c_uint32 * 3),
                ("lds_step", c_uint32 * 3), ("part_step", c_uint32 * 3), ("sstride", c_int64 * 7),
                ("dstride", c_int64 * 7), ("n_boxes", c_int32), ("n_list", c_int32), ("n_tiles", c_uint32),
                ("max_grid", c_uint32), ("bytes_read", c_int64), ("bytes_written", c_int64), ("min_stretch", c_int64),
                ("spv", c_uint32), ("spv_magic", c_uint32), ("spv_shift", c_uint32), ("dpv", c_uint32),
                ("dpv_magic", c_uint32), ("dpv_shift", c_uint32), ("drg_magic", c_uint32), ("drg_shift", c_uint32),
                ("dext_magic", c_uint32 * 3), ("dext_shift", c_uint32 * 3), ("piece_magic", c_uint32 * 3),
                ("piece_shift", c_uint32 * 3), ("tiles_per_box", c_uint32), ("tpb_magic", c_uint32),
                ("tpb_shift", c_uint32), ("pad", c_uint32)]


class RowInfo(ctypes.Structure):
    _fields_ = [("enabled", c_int32), ("dir", c_int32), ("n_outer", c_int32), ("w_log2", c_int32), ("n_log2", c_int32),
                ("r_log2", c_int32), ("vn", c_int32), ("n_pieces", c_int32), ("narrow_count", c_int32),
                ("n_boxes", c_int32), ("n_pieces_total", c_int32), ("n_dev_list", c_int32), ("n_tiles", c_uint32),
                ("tiles_per_box", c_uint32), ("tpb_magic", c_uint32), ("tpb_shift", c_uint32),
                ("general", c_int32), ("w_bytes", c_uint32), ("n_bytes", c_uint32), ("pitch", c_uint32),
                ("cpn", c_uint32), ("cpn_magic", c_uint32), ("cpn_shift", c_uint32), ("wpr", c_uint32),
                ("wpr_magic", c_uint32), ("wpr_shift", c_uint32), ("vw", c_int32),
                ("span", c_int32), ("gran", c_int32), ("chunk_dims", c_int32), ("rpt", c_uint32), ("mct", c_uint32),
                ("slot", c_uint32), ("cbw", c_uint32), ("cbw_magic", c_uint32), ("cbw_shift", c_uint32),
                ("nbm", c_uint32), ("nbm_magic", c_uint32), ("nbm_shift", c_uint32),
                ("wstride", c_int64 * 7), ("nstride", c_int64 * 7), ("src_shard_bytes", c_int64),
                ("dst_shard_bytes", c_int64), ("dest_major", c_int32), ("dm_count", c_uint32), ("dm_magic", c_uint32),
                ("dm_shift", c_uint32), ("chunk_tiles", c_uint32), ("src_tiles", c_uint32), ("max_grid", c_uint32),
                ("pad2", c_uint32), ("dm_fanout", c_uint32), ("dm_groups", c_uint32), ("rpt_magic", c_uint32),
                ("rpt_shift", c_uint32)]


_lib = None


def lib():
    """The loaded library; built with paper_2112_01075_amd/build.py (hipcc, gfx950)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise ImportError("libredist.so is not built: run `python -m paper_2112_01075_amd.build` "
                              "(there is no fallback path)")
        L = ctypes.CDLL(_LIB_PATH)
        P = c_void_p
        L.redist_plan_create.argtypes = [POINTER(_Mesh), POINTER(_Type), POINTER(_Type), c_int32, c_uint32, POINTER(P)]
        L.redist_plan_create.restype = c_int32
        L.redist_plan_destroy.argtypes = [P]
        L.redist_plan_destroy.restype = None
        L.redist_plan_create_cached.argtypes = L.redist_plan_create.argtypes
        L.redist_plan_create_cached.restype = c_int32
        L.redist_options_init.argtypes, L.redist_options_init.restype = [POINTER(Options)], None
        L.redist_plan_create_ex.argtypes = [POINTER(_Mesh), POINTER(_Type), POINTER(_Type), c_int32, c_uint32,
                                            POINTER(Options), c_int32, POINTER(P)]
        L.redist_plan_create_ex.restype = c_int32
        L.redist_plan_cache_clear.argtypes, L.redist_plan_cache_clear.restype = [], None
        L.redist_plan_cache_size.argtypes, L.redist_plan_cache_size.restype = [], c_int32
        for name in ("num_devices", "rank", "mode", "num_steps", "search_limits_hit"):
            f = getattr(L, "redist_plan_" + name)
            f.argtypes, f.restype = [P], c_int32
        L.redist_plan_step.argtypes = [P, c_int32, POINTER(c_int32), POINTER(c_int32), POINTER(c_int32),
                                       POINTER(c_int64), POINTER(c_int64)]
        L.redist_plan_step.restype = c_int32
        L.redist_plan_step_offsets.argtypes = [P, c_int32, POINTER(c_int64)]
        L.redist_plan_step_offsets.restype = c_int32
        L.redist_plan_step_peers.argtypes = [P, c_int32, POINTER(c_int32)]
        L.redist_plan_step_peers.restype = c_int32
        for name in ("cost_elems", "weak_cost_elems", "height_elems", "bound_elems", "peak_live_bytes_per_shard",
                     "workspace_bytes", "footprint_bytes_per_shard", "predicted_ns"):
            f = getattr(L, "redist_plan_" + name)
            f.argtypes, f.restype = [P], c_int64
        L.redist_plan_algorithmic_bytes.argtypes = [P, c_int32]
        L.redist_plan_algorithmic_bytes.restype = c_int64
        L.redist_plan_step_kernel.argtypes = [P, c_int32]
        L.redist_plan_step_kernel.restype = c_char_p
        L.redist_plan_num_ops.argtypes, L.redist_plan_num_ops.restype = [P], c_int32
        L.redist_plan_op_last_step.argtypes, L.redist_plan_op_last_step.restype = [P, c_int32], c_int32
        L.redist_plan_op_info.argtypes, L.redist_plan_op_info.restype = [P, c_int32, POINTER(OpInfo)], c_int32
        L.redist_plan_op_tables.argtypes = [P, c_int32, POINTER(Box), POINTER(c_int32)]
        L.redist_plan_op_tables.restype = c_int32
        L.redist_plan_op_row_info.argtypes, L.redist_plan_op_row_info.restype = [P, c_int32, POINTER(RowInfo)], c_int32
        L.redist_plan_op_row_tables.argtypes = [P, c_int32, POINTER(RowBox), POINTER(Piece), POINTER(c_int32)]
        L.redist_plan_op_row_tables.restype = c_int32
        L.redist_plan_op_cell_info.argtypes, L.redist_plan_op_cell_info.restype = [P, c_int32, POINTER(CellInfo)], c_int32
        L.redist_plan_op_cell_tables.argtypes = [P, c_int32, POINTER(CellBox), POINTER(c_int32)]
        L.redist_plan_op_cell_tables.restype = c_int32
        L.redist_plan_prepare.argtypes = [P]
        L.redist_plan_prepare.restype = c_int32
        L.redist_execute.argtypes = [P, POINTER(c_void_p), POINTER(c_void_p), c_void_p, c_void_p]
        L.redist_execute.restype = c_int32
        L.redist_execute_range.argtypes = [P, POINTER(c_void_p), POINTER(c_void_p), c_void_p, c_void_p, c_int32, c_int32]
        L.redist_execute_range.restype = c_int32
        L.redist_execute_static.argtypes = [P, POINTER(c_void_p), POINTER(c_void_p), c_void_p]
        L.redist_execute_static.restype = c_int32
        L.redist_plan_static_fits.argtypes, L.redist_plan_static_fits.restype = [P], c_int32
        L.redist_plan_op_output.argtypes = [P, c_int32, POINTER(c_int64), POINTER(c_int64)]
        L.redist_plan_op_output.restype = c_int32
        L.redist_copy_baseline.argtypes = [c_void_p, c_void_p, c_int64, c_void_p]
        L.redist_copy_baseline.restype = c_int32
        L.redist_status_string.argtypes = [c_int32]
        L.redist_status_string.restype = c_char_p
        _lib = L
    return _lib


def _check(status):
    if status != 0:
        raise RedistError(status, lib().redist_status_string(status).decode())


def parse_type(text, mesh_axes, mesh_sizes=None):
    """"[32{a}64, 24{b}48]" -> (global_shape, [[axis ids of dim 0], ...]); a bare number is an untiled dim.
    mesh_axes: axis names in declaration order.  Syntax only: tile sizes are re-derived by the library; when
    mesh_sizes is given, a written tile size that contradicts them is an error."""
    inner = text.strip()
    if not (inner.startswith("[") and inner.endswith("]")):
        raise ValueError("type must look like [c{axes}n, ...]: %r" % (text,))
    gshape, axes = [], []
    for tok in re.findall(r"\d+\s*\{[^}]*\}\s*\d+|\d+", inner[1:-1]):
        m = re.fullmatch(r"(\d+)\s*\{([^}]*)\}\s*(\d+)", tok)
        if m:
            names = [a.strip().strip("\"'") for a in m.group(2).split(",") if a.strip()]
            gshape.append(int(m.group(3)))
            axes.append([list(mesh_axes).index(n) for n in names])
            if mesh_sizes is not None:
                tiles = 1
                for a in axes[-1]:
                    tiles *= int(mesh_sizes[a])
                if int(m.group(1)) * tiles != gshape[-1]:
                    raise ValueError("tile size %s of %r does not match the mesh: %d tiles of a dimension of %d"
                                     % (m.group(1), tok, tiles, gshape[-1]))
        else:
            gshape.append(int(tok))
            axes.append([])
    return gshape, axes


def _c_type(gshape, axes):
    flat = [a for dim in axes for a in dim]
    g = (c_int64 * len(gshape))(*gshape)
    n = (c_int32 * len(gshape))(*[len(d) for d in axes])
    f = (c_int32 * max(1, len(flat)))(*flat) if flat else (c_int32 * 1)(0)
    t = _Type(len(gshape), g, n, f)
    t._keep = (g, n, f)
    return t


class Plan:
    """redist_plan* with its getters.  Create through redist_plan()."""

    def __init__(self, handle):
        self._h = handle

    def __del__(self):
        h, self._h = getattr(self, "_h", None), None
        if h and _lib is not None:
            _lib.redist_plan_destroy(h)

    num_devices = property(lambda s: lib().redist_plan_num_devices(s._h))
    rank = property(lambda s: lib().redist_plan_rank(s._h))
    mode = property(lambda s: lib().redist_plan_mode(s._h))
    num_steps = property(lambda s: lib().redist_plan_num_steps(s._h))
    search_limits_hit = property(lambda s: lib().redist_plan_search_limits_hit(s._h))
    cost_elems = property(lambda s: lib().redist_plan_cost_elems(s._h))
    weak_cost_elems = property(lambda s: lib().redist_plan_weak_cost_elems(s._h))
    height_elems = property(lambda s: lib().redist_plan_height_elems(s._h))
    bound_elems = property(lambda s: lib().redist_plan_bound_elems(s._h))
    peak_live_bytes_per_shard = property(lambda s: lib().redist_plan_peak_live_bytes_per_shard(s._h))
    workspace_bytes = property(lambda s: lib().redist_plan_workspace_bytes(s._h))
    footprint_bytes_per_shard = property(lambda s: lib().redist_plan_footprint_bytes_per_shard(s._h))
    predicted_ns = property(lambda s: lib().redist_plan_predicted_ns(s._h))
    static_fits = property(lambda s: lib().redist_plan_static_fits(s._h) == 1)

    def op_output(self, k):
        """(byte offset in the workspace, bytes between shards) of the intermediate launch k writes."""
        off, stride = c_int64(), c_int64()
        _check(lib().redist_plan_op_output(self._h, k, off, stride))
        return off.value, stride.value

    def algorithmic_bytes(self, which):
        return lib().redist_plan_algorithmic_bytes(self._h, which)

    def step(self, k):
        kind, di, dj, f = c_int32(), c_int32(), c_int32(), c_int64()
        shape = (c_int64 * self.rank)()
        _check(lib().redist_plan_step(self._h, k, kind, di, dj, f, shape))
        return {"kind": STEP_NAMES[kind.value], "dim_i": di.value, "dim_j": dj.value, "factor": f.value,
                "shape_after": tuple(shape)}

    def steps(self):
        return [self.step(k) for k in range(self.num_steps)]

    def step_offsets(self, k):
        """Base offset per device after step k (k = -1: the source assignment)."""
        nd, r = self.num_devices, self.rank
        buf = (c_int64 * (nd * r))()
        _check(lib().redist_plan_step_offsets(self._h, k, buf))
        return [tuple(buf[d * r:(d + 1) * r]) for d in range(nd)]

    def step_peers(self, k):
        st = self.step(k)
        nd = self.num_devices
        n = nd * st["factor"] if st["kind"] in ("allgather", "alltoall") else nd
        buf = (c_int32 * n)()
        _check(lib().redist_plan_step_peers(self._h, k, buf))
        return list(buf)

    def step_kernel(self, k):
        return lib().redist_plan_step_kernel(self._h, k).decode()

    num_ops = property(lambda s: lib().redist_plan_num_ops(s._h))

    def op_last_step(self, k):
        """Index of the last plan step that launch k carries out (-1 for the identity launch of an empty plan)."""
        return lib().redist_plan_op_last_step(self._h, k)

    def op(self, k):
        """(OpInfo, [Box...], [destination shard indices]) of kernel launch k."""
        info = OpInfo()
        _check(lib().redist_plan_op_info(self._h, k, ctypes.byref(info)))
        boxes = (Box * max(1, info.n_boxes))()
        dl = (c_int32 * max(1, info.n_dst_list))()
        _check(lib().redist_plan_op_tables(self._h, k, boxes, dl))
        return info, list(boxes)[:info.n_boxes], list(dl)[:info.n_dst_list]

    def row_op(self, k):
        """(RowInfo, [RowBox...], [Piece...], [shard indices]) of launch k; RowInfo.enabled == 0 if generic."""
        info = RowInfo()
        _check(lib().redist_plan_op_row_info(self._h, k, ctypes.byref(info)))
        boxes = (RowBox * max(1, info.n_boxes))()
        pieces = (Piece * max(1, info.n_pieces_total))()
        dl = (c_int32 * max(1, info.n_dev_list))()
        _check(lib().redist_plan_op_row_tables(self._h, k, boxes, pieces, dl))
        return info, list(boxes)[:info.n_boxes], list(pieces)[:info.n_pieces_total], list(dl)[:info.n_dev_list]

    def cell_op(self, k):
        """(CellInfo, [CellBox...], [list entries]) of launch k; CellInfo.enabled == 0 unless the launch is cell-staged."""
        info = CellInfo()
        _check(lib().redist_plan_op_cell_info(self._h, k, ctypes.byref(info)))
        boxes = (CellBox * max(1, info.n_boxes))()
        dl = (c_int32 * max(1, info.n_list))()
        _check(lib().redist_plan_op_cell_tables(self._h, k, boxes, dl))
        return info, list(boxes)[:info.n_boxes], list(dl)[:info.n_list]

    def prepare(self):
        _check(lib().redist_plan_prepare(self._h))


def redist_plan(mesh, src_type, dst_type, elem_size, mode=MODE_STEPWISE, cached=False, options=None):
    """mesh: {axis name: size} in declaration order; types as text or (global_shape, axes-per-dim).
    cached=True: equal arguments share one plan (redist_plan_create_cached); options: an Options (redist_plan_create_ex)."""
    names = list(mesh.keys())
    sizes = (c_int64 * len(names))(*[int(mesh[n]) for n in names])
    cm = _Mesh(len(names), sizes)
    msz = [int(mesh[n]) for n in names]
    s = parse_type(src_type, names, msz) if isinstance(src_type, str) else src_type
    d = parse_type(dst_type, names, msz) if isinstance(dst_type, str) else dst_type
    cs, cd = _c_type(*s), _c_type(*d)
    out = c_void_p()
    if options is not None:
        _check(lib().redist_plan_create_ex(ctypes.byref(cm), ctypes.byref(cs), ctypes.byref(cd), int(elem_size), int(mode),
                                           ctypes.byref(options), 1 if cached else 0, ctypes.byref(out)))
        return Plan(out)
    create = lib().redist_plan_create_cached if cached else lib().redist_plan_create
    _check(create(ctypes.byref(cm), ctypes.byref(cs), ctypes.byref(cd), int(elem_size), int(mode), ctypes.byref(out)))
    return Plan(out)


def redist_plan_cache_clear():
    lib().redist_plan_cache_clear()


def redist_plan_cache_size():
    return lib().redist_plan_cache_size()


def _ptr(x):
    return int(x.data_ptr()) if hasattr(x, "data_ptr") else int(x)


def redist_execute(plan, src_shards, dst_shards, workspace=None, stream=None):
    """Enqueue the plan.  src_shards / dst_shards: device tensors (or raw device pointers), one per shard in
    shard order; workspace: device tensor / pointer of plan.workspace_bytes bytes; stream: hipStream_t as int
    (default: torch's current stream if torch tensors were passed, else the null stream)."""
    nd = plan.num_devices
    if len(src_shards) != nd or len(dst_shards) != nd:
        raise ValueError("need one source and one destination shard per device")
    sp = (c_void_p * nd)(*[_ptr(t) for t in src_shards])
    dp = (c_void_p * nd)(*[_ptr(t) for t in dst_shards])
    if stream is None and hasattr(src_shards[0], "data_ptr"):
        import torch
        stream = torch.cuda.current_stream().cuda_stream
    ws = None if workspace is None else _ptr(workspace)
    _check(lib().redist_execute(plan._h, sp, dp, ws, stream))


def _marshal(plan, src_shards, dst_shards, stream):
    nd = plan.num_devices
    for shards in (src_shards, dst_shards):
        if shards is not None and len(shards) != nd:
            raise ValueError("need one source and one destination shard per device")
    sp = None if src_shards is None else (c_void_p * nd)(*[_ptr(t) for t in src_shards])
    dp = None if dst_shards is None else (c_void_p * nd)(*[_ptr(t) for t in dst_shards])
    some = src_shards if src_shards is not None else dst_shards
    if stream is None and some is not None and hasattr(some[0], "data_ptr"):
        import torch
        stream = torch.cuda.current_stream().cuda_stream
    return sp, dp, stream


def redist_execute_range(plan, src_shards, dst_shards, workspace, op_begin, op_end, stream=None):
    """Launches op_begin <= k < op_end only (redist_execute_range); shards the range does not touch may be None."""
    sp, dp, stream = _marshal(plan, src_shards, dst_shards, stream)
    ws = None if workspace is None else _ptr(workspace)
    if stream is None and workspace is not None and hasattr(workspace, "data_ptr"):
        import torch
        stream = torch.cuda.current_stream().cuda_stream
    _check(lib().redist_execute_range(plan._h, sp, dp, ws, stream, int(op_begin), int(op_end)))


def redist_execute_static(plan, src_shards, dst_shards, stream=None):
    """redist_execute without workspace, preparation or any allocation (redist_execute_static)."""
    sp, dp, stream = _marshal(plan, src_shards, dst_shards, stream)
    _check(lib().redist_execute_static(plan._h, sp, dp, stream))


class BoundCall:
    """redist_execute with its arguments marshalled once (pointer arrays built at construction), for
    callers that re-issue the same redistribution many times; calling it only crosses the C-ABI."""

    def __init__(self, plan, src_shards, dst_shards, workspace=None, stream=None):
        nd = plan.num_devices
        if len(src_shards) != nd or len(dst_shards) != nd:
            raise ValueError("need one source and one destination shard per device")
        self._keep = (plan, src_shards, dst_shards, workspace)
        self._sp = (c_void_p * nd)(*[_ptr(t) for t in src_shards])
        self._dp = (c_void_p * nd)(*[_ptr(t) for t in dst_shards])
        self._ws = None if workspace is None else _ptr(workspace)
        if stream is None and hasattr(src_shards[0], "data_ptr"):
            import torch
            stream = torch.cuda.current_stream().cuda_stream
        self._stream = stream
        self._h = plan._h
        self._fn = lib().redist_execute

    def __call__(self):
        status = self._fn(self._h, self._sp, self._dp, self._ws, self._stream)
        if status != 0:
            _check(status)


def redist_copy_baseline(dst, src, nbytes, stream=None):
    if stream is None and hasattr(src, "data_ptr"):
        import torch
        stream = torch.cuda.current_stream().cuda_stream
    _check(lib().redist_copy_baseline(_ptr(dst), _ptr(src), int(nbytes), stream))
