/* redist -- type-directed array redistribution on a virtual device mesh (gfx950 / MI355X).
 *
 * C-ABI boundary of the library.  A multi-dimensional array whose dimensions are tiled over the
 * axes of a device mesh is converted from a source distributed type to a target one by a
 * synthesised sequence of dynslice / allgather / alltoall / allpermute steps
 * (arXiv 2112.01075).  The mesh is virtual: every device's local tile ("shard") is a buffer in the
 * one GPU's memory, and each collective is an index-mapped copy between shard buffers.
 *
 * Conventions
 *   - Mesh axes are identified by their index in redist_mesh.axis_size (declaration order).
 *   - A distributed type lists, for every array dimension, the axes tiling it in MINOR-TO-MAJOR
 *     order (fastest-changing first), as in Sec. 2.1 of the paper.  The local tile size of a
 *     dimension is global_shape[t] / product(sizes of its axes).
 *   - Shard index of a mesh coordinate = row-major index over the axes in declaration order,
 *     LAST axis fastest.  Shard k is a dense row-major array of the type's local shape whose
 *     first element is global element T[[type]](coordinate k)  (Fig. "Base offset maps").
 *   - Elements are opaque blocks of elem_size bytes; nothing is computed on them, so results are
 *     bit-exact.
 *
 * Ownership: the caller owns every shard buffer and the workspace.  A plan owns host memory and,
 * after redist_plan_prepare, a few KiB..MiB of device memory holding its copy descriptors; both
 * are released by redist_plan_destroy.  Pointer arrays passed to redist_execute are HOST arrays
 * of DEVICE pointers; they are read during the call and not retained.
 *
 * Errors: every entry point reports through redist_status; nothing aborts or throws across the
 * boundary; output arguments are untouched on failure.
 */
#ifndef REDIST_H
#define REDIST_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  REDIST_OK = 0,
  REDIST_ERR_NULL = 1,            /* a required pointer is null */
  REDIST_ERR_BAD_MESH = 2,        /* no axes, axis size < 1, or more than REDIST_MAX_DEVICES devices */
  REDIST_ERR_ILL_FORMED = 3,      /* violates wf-dim / wf-type (Fig. "Well-formedness rules") */
  REDIST_ERR_GLOBAL_MISMATCH = 4, /* globaltype(src) != globaltype(dst)  (Sec. 2.5) */
  REDIST_ERR_BAD_ELEM_SIZE = 5,   /* elem_size not in {1,2,4,8,16} */
  REDIST_ERR_WORKSPACE = 6,       /* plan needs a workspace and none was given */
  REDIST_ERR_HIP = 7,             /* a HIP runtime call or launch failed */
  REDIST_ERR_INTERNAL = 8,        /* planner self-check failed */
  REDIST_ERR_BAD_ARG = 9,         /* index / mode / size out of range */
  REDIST_ERR_UNSUPPORTED = 10,    /* valid problem outside the executor's limits */
  REDIST_ERR_SEARCH_BUDGET = 11   /* the planner's search limits were exhausted before any plan was found */
} redist_status;

#define REDIST_MAX_RANK 8
#define REDIST_MAX_DEVICES 4096
/* redist_execute passes shard pointers as kernel arguments up to this many devices; larger meshes go
 * through a pointer table in the plan's device memory, rewritten on every call by small kernels on the
 * caller's stream (so one such plan must not be executed on two streams at the same time). */
#define REDIST_MAX_EXEC_DEVICES 128

/* Mesh H = {axis 0 : axis_size[0], ...}  (Fig. "Meshes, distributed types, and meta-functions"). */
typedef struct {
  int32_t n_axes;
  const int64_t* axis_size;
} redist_mesh;

/* Distributed type [d_0..d_{rank-1}], d_t = c_t{axes_t}global_shape[t].
 * axes_flat holds the axis ids of dim 0, then dim 1, ...; n_axes_of_dim[t] of them belong to dim t,
 * each group in minor-to-major order. */
typedef struct {
  int32_t rank;
  const int64_t* global_shape;
  const int32_t* n_axes_of_dim;
  const int32_t* axes_flat;
} redist_type;

typedef struct redist_plan redist_plan; /* opaque; immutable after creation; may be shared by threads */

/* How the plan is carried out. */
enum {
  REDIST_MODE_STEPWISE = 0, /* the synthesised normal-form sequence of collectives: one kernel per step, except that a
                             * run of consecutive dynslices and a run of consecutive allgathers (the prefix and the
                             * suffix of the normal form, Sec. 4.3) are each one kernel: fusing allgathers is the
                             * optimisation Sec. 8 names when it discusses problem P4 of the adversarial table; and
                             * the run of dynslices shares the kernel of the step (or run of allgathers) after it:
                             * slicing is local (Sec. 4.1), the next collective reads the part of each tile the
                             * slice keeps.  redist_plan_num_ops / redist_plan_op_last_step tell which steps a
                             * kernel covers */
                            /* ... likewise the single allpermute of the normal form shares the kernel of the
                             * alltoall before it (else of the allgathers after it): on a virtual mesh it only says
                             * which shard a tile is written to */
  REDIST_MODE_FUSED = 1,    /* one pass: every destination shard gathers straight from the source shards */
  REDIST_MODE_NAIVE = 2,    /* Eq. (2): allgather every dimension, then dynslice (baseline; breaks the bound) */
  REDIST_MODE_AUTO = 3      /* latency-aware choice between STEPWISE and FUSED (the paper's cost model counts
                             * transferred elements only; its discussion of the adversarial table, Sec. 8, names a
                             * latency-aware model as future work).  Both plans are made -- the stepwise one with
                             * a latency term in its search, see redist_options.step_latency_elems, which AUTO sets
                             * from the two constants below unless the caller set it -- and the one with the smaller
                             * predicted time, sum over its launches of (launch latency + bytes moved / bandwidth),
                             * is kept; a tie keeps the collective sequence.  redist_plan_mode tells which one it is,
                             * redist_plan_predicted_ns the prediction.  On a virtual mesh the one-pass gather never
                             * moves more bytes nor takes more launches than the sequence, so AUTO picks FUSED unless
                             * the sequence is one launch of the same bytes. */
};

/* Step kinds reported by redist_plan_step. */
enum {
  REDIST_STEP_DYNSLICE = 0,
  REDIST_STEP_ALLGATHER = 1,
  REDIST_STEP_ALLTOALL = 2,
  REDIST_STEP_ALLPERMUTE = 3,
  REDIST_STEP_FUSED = 4
};

/* Which byte count redist_plan_algorithmic_bytes returns. */
enum {
  REDIST_BYTES_READ_MIN = 0,     /* every distinct global element once:      globalsize * B          */
  REDIST_BYTES_READ_LOGICAL = 1, /* every written element loaded once:       ndev * localsize(dst)*B */
  REDIST_BYTES_WRITE = 2,        /* every destination shard written once:    ndev * localsize(dst)*B */
  REDIST_BYTES_MOVED_BY_PLAN = 3 /* read+write summed over this plan's steps                         */
};

/* Synthesise a plan for redistribute(src -> dst) over mesh  (the memory-constrained problem of
 * Sec. 4.3 / 6.2: prime-factor the mesh, shortest path over weak types with the transfer cost
 * model, lowering to device-level collectives with at most one allpermute, hoisted in front of
 * the trailing allgathers -- Secs. 3, 5, 6, 7).  Host only; never touches the GPU.
 * mesh/src/dst are read during the call only.  On success *out receives a new plan. */
redist_status redist_plan_create(const redist_mesh* mesh, const redist_type* src, const redist_type* dst,
                                 int32_t elem_size, uint32_t mode, redist_plan** out);
void redist_plan_destroy(redist_plan* plan);

/* How a plan is lowered to kernel launches.  redist_options_init fills in the defaults, which are the measured
 * choices and what redist_plan_create uses; the other settings exist for A/B measurements and so that tests reach a
 * code path on a small problem.  None of them changes the result or the plan's step list, cost or height -- except
 * step_latency_elems, which changes which step list the search prefers (see there).  Options are part of a plan's
 * identity: the plan cache keys on them. */
typedef struct {
  uint32_t struct_size;          /* sizeof(redist_options), set by redist_options_init */
  int32_t merge_runs;            /* 1: a run of dynslices / of allgathers is one launch, and a run of dynslices shares
                                  *    the launch of the step after it (stepwise mode; see REDIST_MODE_STEPWISE) */
  int32_t fold_permute;          /* 1: the allpermute shares the launch of the alltoall before it, else of the
                                  *    allgathers after it (needs merge_runs) */
  int32_t lds_staging;           /* 1: steps on the contiguous dimension go through LDS; 2: the same, but boxes that leave
                                  *    gaps in the destination are not cut and sorted by destination address; 0: never */
  int32_t span_form;             /* 1: ... in the span form where rows start off the 16-byte grid */
  int32_t dest_major;            /* 1: destination-major order for large ops that write every tile to several shards */
  int32_t unroll;                /* vectors per thread of the generic kernel: 0 = chosen from the run length, else 1, 2, 4, 8 */
  int64_t dest_major_min_bytes;  /* smallest op that takes destination-major order (default 32 MiB); 0 also drops
                                  * the conditions on piece and stretch sizes */
  uint32_t max_grid;             /* workgroups per launch; an op with more tiles takes several launches.  Default and
                                  * maximum 16777215 (the runtime refuses 2^32 threads per grid dimension) */
  uint32_t reserved;
  /* Latency-aware synthesis (the paper's cost model counts transferred elements only and names a latency term as
   * future work, Sec. 8 on the adversarial table): every step that communicates (allgather, alltoall) costs
   * this many elements more in the shortest-path search, so that small transfers prefer sequences with fewer
   * collectives.  0 (default) is the paper's model.  The cost getters always report the paper's cost. */
  int64_t step_latency_elems;
  /* REDIST_MODE_AUTO and redist_plan_predicted_ns: time of one kernel launch (default 3000 ns) and sustained rate
   * of a large launch (default 5500 GB/s, read + write), as measured on one MI355X with 8 / 32 MiB transfers. */
  int32_t launch_latency_ns;
  int32_t sustained_gbs;
  int32_t dest_major_fanout;     /* destinations a workgroup of the generic destination-major kernel stores its tile to:
                                  * 0 (default) = 2 for ops with up to 8 destinations per tile, else 1; or 1 or 2 */
  int32_t sibling_sources;       /* 1 (default): ops whose destination rows are made of pieces (512 bytes to under 2 MiB)
                                  * from several shards, or whose source rows are dealt out in pieces under 4 KiB, take
                                  * those pieces' boxes in turn, tile by tile or run by run (see redist_op_info);
                                  * 0 never; a larger value: that limit in bytes instead of 2 MiB */
  int32_t cell_form;             /* cell-staged kernel for steps that change the tiling of several inner dims: 1 (default)
                                  * where the other kernels would move stretches under 2 KiB and cells at least double
                                  * them, 0 never, 2 wherever a step qualifies */
} redist_options;
void redist_options_init(redist_options* opt);
/* redist_plan_create with explicit options (null = defaults); cached != 0 shares plans as redist_plan_create_cached does. */
redist_status redist_plan_create_ex(const redist_mesh* mesh, const redist_type* src, const redist_type* dst,
                                    int32_t elem_size, uint32_t mode, const redist_options* opt, int32_t cached,
                                    redist_plan** out);

/* Same as redist_plan_create, but equal arguments share ONE plan (process-wide cache keyed by mesh, both types,
 * elem_size and mode; the synthesis of Sec. 7 runs once per distinct problem).  Every successful call hands out one
 * reference; return it with redist_plan_destroy as usual -- the plan is freed when the cache has dropped it and the
 * last holder has destroyed it.  The cache keeps the 1024 most recently created plans.  Thread-safe.  A shared plan
 * is bound to the device it is first prepared on, like any plan. */
redist_status redist_plan_create_cached(const redist_mesh* mesh, const redist_type* src, const redist_type* dst,
                                        int32_t elem_size, uint32_t mode, redist_plan** out);
/* Drop the cache's references (plans still held elsewhere stay valid) / number of cached plans. */
void redist_plan_cache_clear(void);
int32_t redist_plan_cache_size(void);

/* ---- introspection (host only; total functions; a null plan yields -1 / an error) ---- */
int32_t redist_plan_num_devices(const redist_plan* plan);
int32_t redist_plan_rank(const redist_plan* plan);
int32_t redist_plan_mode(const redist_plan* plan);
int32_t redist_plan_num_steps(const redist_plan* plan);
/* Step k: its kind, the dimensions it acts on (dim_j = -1 unless alltoall; both -1 for allpermute
 * and fused), the factor f (product of the sizes of the axes it moves; 1 for allpermute/fused) and
 * the local tile shape after the step (rank entries).  Any output pointer may be null. */
redist_status redist_plan_step(const redist_plan* plan, int32_t k, int32_t* kind, int32_t* dim_i, int32_t* dim_j,
                               int64_t* factor, int64_t* local_shape_after);
/* Base offset (rank entries per device, device-major) of the tile every physical device holds
 * after step k; k = -1 gives the source assignment T[[src]].  This table is the device assignment
 * <phi, beta> of Sec. 6 reduced to its physically meaningful part beta o phi^-1. */
redist_status redist_plan_step_offsets(const redist_plan* plan, int32_t k, int64_t* out);
/* Device-level description of step k, for replaying it as an MPI-style collective:
 *   dynslice   : out[d]       = index (0..f-1) of the chunk device d keeps            (ndev entries)
 *   allgather, : out[d*f + r] = device of rank r in d's group; ranks follow the      (ndev*f entries)
 *   alltoall     position of the members' tiles along dim_i
 *   allpermute : out[d]       = device whose tile d receives                          (ndev entries)
 *   fused      : not available (REDIST_ERR_BAD_ARG). */
redist_status redist_plan_step_peers(const redist_plan* plan, int32_t k, int32_t* out);
int64_t redist_plan_cost_elems(const redist_plan* plan);      /* Fig. cost model, all steps, elements per device */
int64_t redist_plan_weak_cost_elems(const redist_plan* plan); /* same without the allpermute */
int64_t redist_plan_height_elems(const redist_plan* plan);    /* Def. 4.4: largest local size in the sequence */
int64_t redist_plan_bound_elems(const redist_plan* plan);     /* max(localsize(src), localsize(dst)), Eq. (3) */
/* Which limits of the synthesis were reached while this plan was made (0 = none).  The plan is correct and its weak
 * cost optimal either way; a lowering that needs no allpermute may have gone unseen.  Bit 0: more optimal paths than
 * the 64 that are examined; bit 1: the enumeration of optimal paths stopped at 200000 visits; bit 2: the budget of
 * 4096 simulated lowerings ran out before one without an allpermute was found.  Planning takes a fraction of a
 * millisecond for typical problems and up to a few seconds at the limits the boundary accepts (rank 8 on 4096
 * devices); when not even one path is found within the limits, plan creation returns REDIST_ERR_SEARCH_BUDGET. */
int32_t redist_plan_search_limits_hit(const redist_plan* plan);
/* Largest sum, over the plan's kernel launches, of the tile a launch reads and the tile it writes, in bytes: what a
 * shard holds if every intermediate is freed as soon as the next one exists.  A launch that covers several steps
 * counts its first input and its last output, so it is never more than source tile + target tile, which the caller
 * holds for the whole call anyway. */
int64_t redist_plan_peak_live_bytes_per_shard(const redist_plan* plan);
int64_t redist_plan_workspace_bytes(const redist_plan* plan); /* device bytes redist_execute needs; 0 if none */
/* Predicted duration of one redist_execute call: sum over the plan's launches of (launch latency + bytes the launch
 * reads and writes / sustained rate), with the plan's options.  What REDIST_MODE_AUTO compares. */
int64_t redist_plan_predicted_ns(const redist_plan* plan);
/* What one redist_execute call really keeps resident per shard, in bytes: the caller's source tile and target tile
 * for the whole call, plus the shard's share of the workspace (both ping-pong regions).  At most
 * localsize(src) + localsize(dst) + 2 * bound, and equal to source tile + target tile when the plan is one launch. */
int64_t redist_plan_footprint_bytes_per_shard(const redist_plan* plan);
int64_t redist_plan_algorithmic_bytes(const redist_plan* plan, int32_t which);
/* Name of the HIP kernel of launch k, 0 <= k < redist_plan_num_ops (static string, "" for a bad argument), for
 * matching profiler output. */
const char* redist_plan_step_kernel(const redist_plan* plan, int32_t k);

/* ---- copy descriptors (host only; for checking tools and tests) -------------------------------
 * Each kernel launch of a plan copies a list of boxes.  A box is a strided piece of ONE source
 * shard that lands, at the same offset, in one or several destination shards.  It has up to
 * REDIST_MAX_OUTER outer dims (extents len[], byte strides sstride[] / dstride[] common to the
 * launch) around a contiguous run of run_vecs vectors of vec_bytes bytes.  The kernel cuts a box
 * into tiles of tc x tr vectors (tc * tr <= 256*unroll); tile_first / col_blocks / n_tiles describe that
 * cut and magic[] / shift[] the exact division by len[] (q = mulhi32(n, magic) >> shift, len > 1). */
#define REDIST_MAX_OUTER 7
typedef struct {
  int64_t src_off, dst_off;       /* byte offsets of the box in the source / destination shard */
  int32_t src_dev;                /* source shard index */
  int32_t dst_first, dst_count;   /* range of this box's destinations in the destination list */
  uint32_t run_vecs, rows, tile_first, col_blocks, n_tiles;
  uint32_t len[REDIST_MAX_OUTER];
  uint32_t magic[REDIST_MAX_OUTER];
  uint8_t shift[REDIST_MAX_OUTER];
  uint8_t pad0;
  int32_t dst_dev0;               /* the first destination shard */
  uint32_t cb_magic;              /* exact division by col_blocks (> 1), with cb_shift */
  uint8_t cb_shift;
  uint8_t pad[7];
} redist_box;                     /* 128 bytes */
typedef struct {
  int32_t kind;                   /* REDIST_STEP_* of the kernel entry point */
  int32_t n_boxes, n_dst_list, n_outer, vec_bytes;
  int32_t tc, tr;                 /* tile width (vectors along the run) and height (rows) */
  uint32_t tc_magic, tc_shift;    /* lane e of a tile -> row e / tc, column e % tc */
  /* Destination-major order (ops whose boxes all go to m = dm_count > 1 shards, taken in dm_groups = ceil(m /
   * dm_fanout) groups of dm_fanout consecutive entries of a box's destination list).  tile_first / n_tiles of the
   * boxes count the src_tiles tiles that cover every box once, boxes in source order; the launch has n_tiles =
   * src_tiles * dm_groups workgroups.  Launch index t: chunk c = t / (chunk_tiles*dm_groups); with
   * r = t % (chunk_tiles*dm_groups) and here = min(chunk_tiles, src_tiles - c*chunk_tiles), the workgroup copies
   * tile c*chunk_tiles + r % here to destinations g*dm_fanout .. min(m, (g+1)*dm_fanout) - 1 of that tile's box,
   * g = r / here.  What is in flight writes few shards, a chunk (16 MiB of source) is re-read from L2 once per
   * group.  chunk_tiles is a power of two; dm_magic / dm_shift divide by dm_groups (> 1). */
  int32_t dest_major;
  uint32_t n_tiles, tiles_per_box;
  int32_t unroll;                 /* vectors per thread per tile: a tile holds 256*unroll vectors */
  int32_t nontemporal;            /* streaming (non-temporal) stores; loads too unless dest_major */
  uint32_t tpb_magic, tpb_shift;  /* tile / tiles_per_box = mulhi32(tile, tpb_magic) >> tpb_shift (tiles_per_box > 1) */
  int64_t sstride[REDIST_MAX_OUTER], dstride[REDIST_MAX_OUTER];
  int64_t src_shard_bytes, dst_shard_bytes; /* extent of every source / destination shard buffer */
  uint32_t chunk_tiles, src_tiles;
  uint32_t dm_count, dm_magic, dm_shift;
  uint32_t max_grid;              /* workgroups per launch: the op goes out as ceil(n_tiles / max_grid) launches */
  uint32_t dm_fanout, dm_groups;  /* 1, 1 unless dest_major */
  /* Sibling boxes (sib_count = 1: none): the boxes come in groups of sib_count consecutive boxes of one shape
   * (tiles_per_box tiles each) whose runs follow each other in the destination's rows (or, in ops that are not
   * destination-major, in the source's rows), and their tiles alternate: tile t of the launch's source tiles belongs
   * to group g = t / (sib_count * tiles_per_box); with u = t % (sib_count * tiles_per_box) it is tile u / sib_count
   * of box g * sib_count + u % sib_count.  Consecutive workgroups thereby fill (read) the same rows.  sib_magic /
   * sib_shift divide by sib_count.  Runs wider than a tile keep their 2^sib_inner_log2 tiles together: with
   * q = u >> sib_inner_log2 it is then tile ((q / sib_count) << sib_inner_log2) + (u & (2^sib_inner_log2 - 1)) of
   * box g * sib_count + q % sib_count. */
  uint32_t sib_count, sib_magic, sib_shift, sib_inner_log2;
} redist_op_info;
int32_t redist_plan_num_ops(const redist_plan* plan);      /* kernel launches per redist_execute (>= 1) */
/* The last plan step that launch k carries out (launch k covers the steps after launch k-1's last one up to this
 * one); -1 for the identity launch of an empty plan or a bad argument. */
int32_t redist_plan_op_last_step(const redist_plan* plan, int32_t k);
redist_status redist_plan_op_info(const redist_plan* plan, int32_t k, redist_op_info* out);
/* Where launch k (k < num_ops - 1) leaves its output: shard d of that intermediate starts at byte
 * *region_off + d * *shard_stride of the workspace.  The last launch writes the caller's destination shards
 * (REDIST_ERR_BAD_ARG for it). */
redist_status redist_plan_op_output(const redist_plan* plan, int32_t k, int64_t* region_off, int64_t* shard_stride);
/* boxes: n_boxes entries; dst_list: n_dst_list shard indices.  Either may be null. */
redist_status redist_plan_op_tables(const redist_plan* plan, int32_t k, redist_box* boxes, int32_t* dst_list);

/* Row-complete form of a launch: steps that split or merge the LAST dimension have short common runs,
 * so they are described from their wide side and staged through LDS.  A wide row (W = 2^w_log2 bytes;
 * destination row of a gather, dir 0; source row of a scatter, dir 1) consists of n_pieces pieces of
 * N = 2^n_log2 bytes, each a whole row of a narrow tile (sizes that are not powers of two: general form,
 * w_bytes / n_bytes).  A box covers `rows` wide rows (outer extents
 * len[], strides wstride[] / nstride[] on the two sides); a workgroup handles 2^r_log2 consecutive rows.
 * wide shards: dev_list[wide_first .. +wide_count) (all written by a gather; the first read by a
 * scatter); piece k of a box: pieces[piece_first + k], narrow shards dev_list[dev_first .. +narrow_count). */
typedef struct {
  int64_t wide_off;
  int32_t wide_first, wide_count, piece_first;
  uint32_t rows, tile_first, n_tiles;
  uint32_t len[REDIST_MAX_OUTER];
  uint32_t magic[REDIST_MAX_OUTER];
  uint8_t shift[REDIST_MAX_OUTER];
  uint8_t tpc_shift;
  uint32_t chunk_rows, tpc, tpc_magic;  /* span form: rows of a chunk, virtual chunks per chunk and the reciprocal */
  uint32_t n_vchunks;                   /* span form: virtual chunks of the box; n_tiles = ceil(n_vchunks / mct) */
  uint32_t vrows;                       /* span form: rows per virtual chunk = ceil(chunk_rows / tpc) <= rpt */
  uint8_t pad[12];
} redist_row_box;                 /* 128 bytes */
typedef struct {
  int64_t narrow_off;
  int32_t dev_first, pad;
} redist_piece;                   /* 16 bytes */
typedef struct {
  int32_t enabled;                /* 0: the launch uses the generic boxes above */
  int32_t dir, n_outer, w_log2, n_log2, r_log2, vn, n_pieces, narrow_count;
  int32_t n_boxes, n_pieces_total, n_dev_list;
  uint32_t n_tiles, tiles_per_box, tpb_magic, tpb_shift;
  /* general form (W or N not a power of two): narrow vectors of vn bytes, wide vectors of vw bytes, staged rows pitch bytes
   * apart, cpn = N / vn vectors per piece row, wpr = W / vn vectors per wide row, each with its reciprocal */
  int32_t general;
  uint32_t w_bytes, n_bytes, pitch, cpn, cpn_magic, cpn_shift, wpr, wpr_magic, wpr_shift;
  int32_t vw;                     /* wide-side vector bytes of the general form: 16 or vn; wpr = W / vw */
  /* span form (general = 1, span = 1): rows start at odd multiples of a granule of gran = vn < 16 bytes.  Rows
   * contiguous on both sides form chunks: the innermost outer extent when chunk_dims = n_outer - 1 (then
   * wstride[n_outer-1] = W and nstride[n_outer-1] = N), single rows when chunk_dims = n_outer; the leading
   * chunk_dims extents number the chunks.  A chunk longer than rpt rows is cut into tpc virtual chunks; a tile is
   * up to mct consecutive virtual chunks of a box, each one contiguous span per side.  16-byte aligned blocks
   * of memory cover each span: whole blocks move as vectors, the granules of edge blocks one by one (loads read
   * an edge block whole when it lies inside the shard).  cpn = N / gran; nbm / cbw bound the blocks that cover one
   * piece's / one wide span.  The staging area gives virtual chunk c of a tile the bytes [c*slot, (c+1)*slot) and
   * holds byte s of its wide span at c*slot + (wide offset mod 16) + s. */
  int32_t span, gran, chunk_dims;
  uint32_t rpt, mct, slot, cbw, cbw_magic, cbw_shift, nbm, nbm_magic, nbm_shift;
  int64_t wstride[REDIST_MAX_OUTER], nstride[REDIST_MAX_OUTER];
  int64_t src_shard_bytes, dst_shard_bytes;
  /* destination-major order (as in redist_op_info): the boxes' tiles number src_tiles, the launch
   * has n_tiles = src_tiles * dm_groups workgroups, and launch index t stages tile c*chunk_tiles + r % here for the
   * (r / here)-th group of dm_fanout of the dm_count shards that receive it -- the wide_count shards of its box for a gather, the
   * narrow_count shards of each piece for a scatter.  For a gather, tile l of a whole chunk is taken by launch
   * position (l % (chunk_tiles/8)) * 8 + l / (chunk_tiles/8) of the chunk, i.e. position p stages tile
   * (p % 8) * (chunk_tiles / 8) + p / 8: the workgroups of one XCD (every eighth) take a contiguous eighth of the chunk. */
  int32_t dest_major;
  uint32_t dm_count, dm_magic, dm_shift, chunk_tiles, src_tiles;
  uint32_t max_grid, pad2;        /* as in redist_op_info */
  uint32_t dm_fanout, dm_groups;  /* as in redist_op_info: a workgroup serves dm_fanout consecutive receiving shards,
                                   * n_tiles = src_tiles * dm_groups, dm_magic / dm_shift divide by dm_groups */
  uint32_t rpt_magic, rpt_shift;  /* row-by-row general form: a tile is rpt rows (any number up to 256; r_log2 is the floor
                                   * of its logarithm and not used), rpt_magic / rpt_shift divide by it */
} redist_row_info;
redist_status redist_plan_op_row_info(const redist_plan* plan, int32_t k, redist_row_info* out);
redist_status redist_plan_op_row_tables(const redist_plan* plan, int32_t k, redist_row_box* boxes, redist_piece* pieces,
                                        int32_t* dev_list);

/* Cell-complete form of a launch (enabled = 1; it then takes precedence over the two forms above).  For steps that
 * change the tiling of the last dim and of dims close to it, whose common contiguous stretches are short on both
 * sides whichever side rows are taken from (two shards alternate every 144 bytes in the destination, say).  The
 * innermost n_cell dims are taken whole on both sides -- extent max(source tile, destination tile), tilings nested --
 * so a cell is the whole local extent of ps source tiles (parts) and of pd destination tiles at once; the dim in
 * front of them counts rows.  A workgroup takes rows_per_tile consecutive rows of a box: one contiguous stretch of
 * rows * src_row_bytes bytes of every source part, staged part after part (part s at s * part_pitch), and one
 * contiguous stretch of rows * dst_row_bytes bytes of every destination part, written whole to each of its rep
 * shards.  Source part s of a box is read from shard dev_list[src_first + s], destination part q written to shards
 * dev_list[dst_first + q * rep + j]; both at the box's offsets plus outer index * stride (the last outer extent
 * counts rows; its strides are the row bytes).  Staging address of granule g (gran bytes) of row k of destination
 * part q: dev_list[base_first + q] + k * src_row_bytes + sum over the cell dims, last dim (index 0, in granules)
 * first, of the digit x of g over dext[]: where piece[i] > 0, (x / piece[i]) * part_step[i] + (x % piece[i]) *
 * lds_step[i], else x * lds_step[i]. */
typedef struct {
  int64_t src_off, dst_off;
  int32_t src_first, dst_first;
  uint32_t tile_first, n_tiles, row_tiles, rt_magic;
  uint32_t len[REDIST_MAX_OUTER];
  uint32_t magic[REDIST_MAX_OUTER];
  uint8_t shift[REDIST_MAX_OUTER];
  uint8_t rt_shift;
  uint8_t pad[8];
} redist_cell_box;                /* 112 bytes */
typedef struct {
  int32_t enabled;
  int32_t n_outer, n_cell, ps, pd, rep, vs, vd, gran, base_first;
  uint32_t rows_per_tile, src_row_bytes, dst_row_bytes, part_pitch, drow_gran;
  uint32_t dext[3], piece[3], lds_step[3], part_step[3];
  int64_t sstride[REDIST_MAX_OUTER], dstride[REDIST_MAX_OUTER];
  int32_t n_boxes, n_list;
  uint32_t n_tiles, max_grid;
  int64_t bytes_read, bytes_written;
  int64_t min_stretch;            /* shortest stretch a tile reads or writes per shard, bytes */
  /* vectors of a full tile's stretch of one source / destination part, and the reciprocals the kernel divides by
   * (n / d = (n * magic >> 32) >> shift for d > 1): by spv, dpv, drow_gran, dext[i], piece[i], tiles_per_box */
  uint32_t spv, spv_magic, spv_shift, dpv, dpv_magic, dpv_shift, drg_magic, drg_shift;
  uint32_t dext_magic[3], dext_shift[3], piece_magic[3], piece_shift[3];
  uint32_t tiles_per_box, tpb_magic, tpb_shift, pad;
} redist_cell_info;
redist_status redist_plan_op_cell_info(const redist_plan* plan, int32_t k, redist_cell_info* out);
redist_status redist_plan_op_cell_tables(const redist_plan* plan, int32_t k, redist_cell_box* boxes, int32_t* dev_list);

/* Upload the plan's copy descriptors to the current HIP device (allocates device memory once;
 * synchronous).  redist_execute calls it on first use if the caller did not. */
redist_status redist_plan_prepare(redist_plan* plan);

/* Carry out the plan: enqueue its kernels on hip_stream (a hipStream_t, may be null for the
 * default stream) and return without synchronising.
 *   src_shards / dst_shards : host arrays of ndev device pointers, shard order as above; the
 *                             buffers must not overlap each other or the workspace and must be
 *                             16-byte aligned (REDIST_ERR_BAD_ARG otherwise).
 *   workspace               : device buffer of redist_plan_workspace_bytes() bytes, 256-byte
 *                             aligned; may be null when that is 0.
 * The plan's descriptors live on the device it was prepared on: calling with another current device is
 * REDIST_ERR_UNSUPPORTED.  Launch failures are returned as REDIST_ERR_HIP.
 * On a prepared plan the call only enqueues kernels (no allocation, no copy, no synchronisation), so it may be
 * recorded into a HIP graph by stream capture; the graph then holds the shard pointers of the recorded call. */
redist_status redist_execute(redist_plan* plan, const void* const* src_shards, void* const* dst_shards,
                             void* workspace, void* hip_stream);

/* Launches op_begin <= k < op_end of the plan only (0 <= op_begin < op_end <= num_ops), arguments as for
 * redist_execute: launch 0 reads src_shards, the last launch writes dst_shards, every other input and output is an
 * intermediate in the workspace (redist_plan_op_output).  For checking a plan step by step (the device tables of
 * redist_plan_step_offsets say what every intermediate must hold) and for interleaving other work between the
 * launches.  src_shards / dst_shards may be null when the range does not touch them. */
redist_status redist_execute_range(redist_plan* plan, const void* const* src_shards, void* const* dst_shards,
                                   void* workspace, void* hip_stream, int32_t op_begin, int32_t op_end);

/* redist_execute for callers that must not allocate device memory or cannot provide a workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  The plan need not be prepared and no
 * workspace is passed: the copy descriptors and the intermediates of a multi-launch plan live in a fixed
 * scratch area of REDIST_STATIC_SCRATCH_BYTES bytes that is part of the library's device image (every GPU the
 * library runs on holds one until the process ends).  The call allocates and frees nothing and calls no
 * allocating runtime routine; descriptors reach the scratch area as kernel arguments of small upload kernels on
 * hip_stream, and are uploaded again only when another plan used the area in between.
 *   Limits: at most REDIST_MAX_EXEC_DEVICES devices; descriptors at most REDIST_STATIC_DESC_BYTES; workspace at
 *   most REDIST_STATIC_SCRATCH_BYTES - REDIST_STATIC_DESC_BYTES.  Beyond them: REDIST_ERR_UNSUPPORTED, nothing enqueued
 *   (redist_plan_static_fits tells in advance).
 *   All calls on one GPU share the one area, which keeps the previous call's contents: two calls that overlap in
 *   time on one GPU (different streams, or different threads) race and give undefined results; calls on one stream
 *   are ordered.  Results are those of redist_execute. */
#define REDIST_STATIC_SCRATCH_BYTES (32 * 1024 * 1024)
#define REDIST_STATIC_DESC_BYTES (1024 * 1024)
redist_status redist_execute_static(redist_plan* plan, const void* const* src_shards, void* const* dst_shards,
                                    void* hip_stream);
int32_t redist_plan_static_fits(const redist_plan* plan);   /* 1 / 0; -1 for a null plan */

/* Plain device-to-device copy kernel (16 bytes per lane), the practical bandwidth ceiling the
 * redistribution kernels are compared with.  dst/src are device pointers, 16-byte aligned;
 * bytes must be a multiple of 16. */
redist_status redist_copy_baseline(void* dst, const void* src, int64_t bytes, void* hip_stream);

const char* redist_status_string(redist_status s);

#ifdef __cplusplus
}
#endif
#endif /* REDIST_H */
