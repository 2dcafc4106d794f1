// Lowering of one redistribution step to a list of strided box copies between shard buffers.
//
// Every collective of the paper only changes which tile of the global array a device holds
// (Def. 4.3), so a step is fully described by the device tables before and after it: each
// destination tile is a union of boxes, each box lying inside one source tile.  The same builder
// therefore serves dynslice, allgather, alltoall, allpermute, the fused one-pass gather
// (table T[[src]] -> table T[[dst]]) and the steps of the naive baseline.
#pragma once
#include <cstddef>
#include <cstdint>
#include <vector>

namespace redist {

constexpr int kMaxOuter = 7;  // dims of a box besides its contiguous run

// Device-side box descriptor (also used on the host while building).  128 bytes.
struct alignas(16) DevBox {
  int64_t src_off;      // byte offset of the box's first element in the source shard
  int64_t dst_off;      // byte offset in every destination shard of the box
  int32_t src_dev;      // index into the source pointer table
  int32_t dst_first;    // first entry of this box's destinations in the destination list
  int32_t dst_count;    // number of destination shards receiving identical bytes
  uint32_t run_vecs;    // contiguous run, in vectors of the op's vector width
  uint32_t rows;        // product of the outer extents
  uint32_t tile_first;  // index of the box's first tile among the tiles that cover every box of the op once
  uint32_t col_blocks;  // tiles per row block
  uint32_t n_tiles;     // tiles of this box
  uint32_t len[kMaxOuter];    // outer extents, outermost first
  uint32_t magic[kMaxOuter];  // division by len[k]: q = umulhi(n, magic) >> shift  (n < 2^31, len > 1)
  uint8_t shift[kMaxOuter];
  uint8_t pad0;
  int32_t dst_dev0;     // the first destination shard (saves a dependent table load when it is the only one)
  uint32_t cb_magic;    // division by col_blocks (col_blocks > 1), same scheme as magic[]
  uint8_t cb_shift;
  uint8_t pad[7];
};
static_assert(sizeof(DevBox) == 128, "DevBox layout");  // mirrored by redist_box in the public header
static_assert(offsetof(DevBox, shift) % 4 == 0, "the kernels read shift[] in 32-bit words");

// ---- row-complete ops (LDS-staged) ---------------------------------------------------------------
// When a step splits or merges the LAST (contiguous) dimension, the contiguous runs common to both
// sides are short (down to one element).  Such a step is described from its wide side: a row of W
// bytes of the wide tile (destination of a gather, source of a scatter) consists of P pieces of N
// bytes, each a whole row of some narrow tile.  A workgroup stages R wide rows in LDS so that both
// the wide side (whole rows) and the narrow side (R consecutive narrow rows = R*N contiguous bytes)
// are accessed in long contiguous stretches.
struct alignas(16) DevRowBox {
  int64_t wide_off;         // byte offset of the box's first row in the wide shard(s)
  int32_t wide_first;       // first entry of the wide-side shards in the device list
  int32_t wide_count;       // gather: all of them are written; scatter: the first one is read
  int32_t piece_first;      // first of the box's n_pieces entries in the piece table
  uint32_t rows;            // product of the outer extents
  uint32_t tile_first;      // index of the box's first tile
  uint32_t n_tiles;
  uint32_t len[kMaxOuter];
  uint32_t magic[kMaxOuter];
  uint8_t shift[kMaxOuter];
  uint8_t tpc_shift;
  // span form: the innermost outer dim counts rows that are contiguous on both sides (a chunk);
  // a chunk is cut into tpc tiles
  uint32_t chunk_rows;
  uint32_t tpc;
  uint32_t tpc_magic;       // division by tpc
  uint32_t n_vchunks;       // virtual chunks of the box = chunks * tpc
  uint32_t vrows;           // rows per virtual chunk = ceil(chunk_rows / tpc): a long chunk is cut evenly
  uint8_t pad[12];
};
static_assert(sizeof(DevRowBox) == 128, "DevRowBox layout");
static_assert(offsetof(DevRowBox, shift) % 4 == 0, "the kernels read shift[] in 32-bit words");

struct alignas(16) DevPiece {
  int64_t narrow_off;       // byte offset of the piece's first row in the narrow shard(s)
  int32_t dev_first;        // first of narrow_count narrow-side shards in the device list
  int32_t pad;
};
static_assert(sizeof(DevPiece) == 16, "DevPiece layout");

struct RowOp {
  bool enabled = false;
  int dir = 0;                  // 0: gather (narrow side = source), 1: scatter (narrow side = destination)
  int n_outer = 0;
  int64_t wstride[kMaxOuter];   // byte strides of the outer dims on the wide / narrow side
  int64_t nstride[kMaxOuter];
  int w_log2 = 0, n_log2 = 0;   // W = 2^w_log2 bytes per wide row, N = 2^n_log2 bytes per piece
  int r_log2 = 0;               // R = 2^r_log2 wide rows per tile
  int vn = 16;                  // vector width on the narrow side = min(16, N)
  int n_pieces = 0;             // P = W / N
  int narrow_count = 1;         // narrow-side shards per piece (1 for a gather)
  // General form, for W or N not powers of two: narrow-side vectors of vn bytes, wide-side vw; staged rows
  // `pitch` bytes apart (padded), indices by reciprocal division instead of shifts.
  bool general = false;
  int vw = 16;                  // wide-side vector width of the general form: 16 when rows and offsets allow, else vn
  uint32_t w_bytes = 0, n_bytes = 0, pitch = 0;
  uint32_t cpn = 0, cpn_magic = 0, cpn_shift = 0;   // vectors per piece row, and division by it
  uint32_t wpr = 0, wpr_magic = 0, wpr_shift = 0;   // vectors per wide row, and division by it
  // Span form, for sides that cannot move 16-byte vectors row by row (rows start at odd multiples of the
  // granule `gran` = widest power of two dividing N, W and every offset).  Rows contiguous on both sides
  // form chunks (the innermost outer dim when chunk_dims = n_outer - 1; single rows when chunk_dims =
  // n_outer); a chunk longer than rpt rows is cut into tpc virtual chunks; a tile is up to mct virtual
  // chunks, each one contiguous span per side.  16-byte aligned blocks cover each span (whole blocks move
  // as vectors, the granules of the two edge blocks one by one); the staging area gives each virtual
  // chunk `slot` bytes and holds it in the wide side's byte order, shifted so that aligned blocks of the
  // wide span are aligned in LDS.
  bool span = false;
  int gran = 0;
  int chunk_dims = 0;                               // leading outer dims that number the chunks
  uint32_t rpt = 0;                                 // rows per virtual chunk, at most; row-by-row general form: rows per tile
  uint32_t rpt_magic = 0, rpt_shift = 0;            // ... and division by it (general form)
  uint32_t mct = 0;                                 // virtual chunks per tile, at most
  uint32_t slot = 0;                                // staging bytes per virtual chunk = 16 * cbw
  uint32_t cbw = 0, cbw_magic = 0, cbw_shift = 0;   // upper bound of blocks per wide span, and division by it
  uint32_t nbm = 0, nbm_magic = 0, nbm_shift = 0;   // upper bound of blocks per piece span, and division by it
  int64_t wide_shard_bytes = 0, narrow_shard_bytes = 0;  // whole blocks are read only inside the shard
  uint32_t tiles_per_box = 0, tpb_magic = 0, tpb_shift = 0, n_tiles = 0;
  uint32_t max_grid = 16777215u;                    // an op with more tiles takes several launches
  // Destination-major order, as for the generic body (see CopyOp).  A tile is staged once
  // per shard that receives it (m = wide_count of every box for a gather, narrow_count for a scatter): launch
  // index = (chunk of chunk_tiles tiles, which of the m shards, tile of the chunk), boxes in source order.
  bool dest_major = false;
  uint32_t dm_count = 1, dm_magic = 0, dm_shift = 0, chunk_tiles = 0, src_tiles = 0;
  uint32_t dm_fanout = 1, dm_groups = 1;   // as in CopyOp: shards per workgroup, and groups of that many (n_tiles = src_tiles * dm_groups)
  int64_t min_stretch = 0;                 // shortest contiguous stretch a full tile reads or writes per shard, bytes
  std::vector<DevRowBox> boxes;
  std::vector<DevPiece> pieces;
  std::vector<int32_t> dev_list;
  int64_t bytes_read = 0, bytes_written = 0;
};

// ---- cell-complete ops (LDS-staged, several dims) -----------------------------------------------
// A step that changes the tiling of the last dimension AND of dims close to it leaves short stretches on both sides
// whatever side the rows are taken from: 16-byte pieces of 32-byte rows of which only 9 are consecutive in the
// destination (144 bytes, the next 144 come from another shard), say.  Partly written 32-byte sectors cost a second
// write of the sector (measured: 1.14 and 1.36 times the algorithmic bytes written, 1.8 and 2.0 TB/s on two such
// problems).  Such a step is described by CELLS instead: the innermost n_cell dims (the cell dims) are taken whole
// on both sides -- extent max(source tile, destination tile), tilings nested -- so that a cell is the whole local
// extent of `ps` source tiles (parts) and of `pd` destination tiles at once.  The dim in front of them counts ROWS; a
// workgroup takes rows_per_tile consecutive rows: one contiguous stretch of every source part, staged in LDS part
// after part, and one contiguous stretch of every destination part, written whole.  The dims in front of the row dim
// are outer dims as for the other ops (boxes = intersections of source and destination tiles on them).
constexpr int kMaxCellDims = 3;
constexpr int kCellTileBytes = 16384;  // LDS staging area per workgroup
constexpr int kCellMaxParts = 64;      // source parts per cell; destination parts times replicas per cell

struct alignas(16) DevCellBox {
  int64_t src_off;            // byte offset of the box's first row in every source part
  int64_t dst_off;            // ... in every destination part
  int32_t src_first;          // dev_list[src_first + s]: shard read for source part s
  int32_t dst_first;          // dev_list[dst_first + q * rep + j]: j-th shard written for destination part q
  uint32_t tile_first;        // index of the box's first tile
  uint32_t n_tiles;
  uint32_t row_tiles;         // tiles along the row dim = ceil(len[n_outer-1] / rows_per_tile)
  uint32_t rt_magic;          // division by row_tiles (row_tiles > 1)
  uint32_t len[kMaxOuter];    // outer extents, outermost first; the last one counts rows
  uint32_t magic[kMaxOuter];
  uint8_t shift[kMaxOuter];
  uint8_t rt_shift;
  uint8_t pad[8];
};
static_assert(sizeof(DevCellBox) == 112, "DevCellBox layout");  // mirrored by redist_cell_box in the public header

struct CellOp {
  bool enabled = false;
  int n_outer = 0;                 // outer dims in use, the last of them the row dim (extent 1 when there is none)
  int64_t sstride[kMaxOuter];      // byte strides of the outer dims on the source / destination side;
  int64_t dstride[kMaxOuter];      // those of the row dim are src_row_bytes / dst_row_bytes
  int n_cell = 0;
  int ps = 1, pd = 1, rep = 1;     // source parts, destination parts, shards written per destination part
  int vs = 16, vd = 16, gran = 16; // vector widths of the two sides; granule = widest power of two (<= 16) dividing
                                   // every piece of the last dim: what the staging area is addressed in
  uint32_t rows_per_tile = 1;
  uint32_t src_row_bytes = 0, dst_row_bytes = 0;   // bytes of one row of a source part / of a destination part
  uint32_t part_pitch = 0;         // staging bytes per source part: rows_per_tile * src_row_bytes rounded up to 16
  uint32_t spv = 0, spv_magic = 0, spv_shift = 0;  // vectors of a full tile's stretch of one source part, reciprocal
  uint32_t dpv = 0, dpv_magic = 0, dpv_shift = 0;  // ... of one destination part
  uint32_t drow_gran = 0, drg_magic = 0, drg_shift = 0;   // granules per destination row, reciprocal
  // Granule g of a destination row -> digits over dext[0 .. n_cell) (last fastest; the last dim counts granules).
  // Along a dim with several source parts (piece[t] > 0: the source tile's extent there) digit x lies in part
  // x / piece[t] at x % piece[t]; staging address = part_base[q] + row * src_row_bytes + sum(part * part_step[t] +
  // x * lds_step[t]).
  uint32_t dext[kMaxCellDims], dext_magic[kMaxCellDims], dext_shift[kMaxCellDims];
  uint32_t piece[kMaxCellDims], piece_magic[kMaxCellDims], piece_shift[kMaxCellDims];
  uint32_t lds_step[kMaxCellDims], part_step[kMaxCellDims];
  int32_t base_first = 0;          // dev_list[base_first + q]: staging byte offset of destination part q's first granule
  uint32_t tiles_per_box = 0, tpb_magic = 0, tpb_shift = 0, n_tiles = 0;
  uint32_t max_grid = 16777215u;
  std::vector<DevCellBox> boxes;
  std::vector<int32_t> dev_list;
  int64_t bytes_read = 0, bytes_written = 0;
  int64_t min_stretch = 0;         // shortest contiguous stretch a full tile reads or writes per shard, in bytes
};

constexpr int kRowTileBytes = 16384;   // LDS staging area per workgroup
constexpr int kRowMaxPtrs = 512;       // narrow-side base pointers cached in LDS (P * narrow_count; span form: times chunks per tile)
constexpr int kRowMaxChunks = 64;      // virtual chunks per tile of the span form

struct CopyOp {
  int kind = 0;                 // StepKind, selects the kernel entry point
  RowOp row;                    // when row.enabled the LDS-staged kernel carries out the op
  CellOp cell;                  // when cell.enabled the cell-staged kernel does (it then takes precedence)
  int n_outer = 0;              // outer dims in use
  int64_t sstride[kMaxOuter];   // byte strides of the outer dims in a source shard
  int64_t dstride[kMaxOuter];   // ... in a destination shard
  int vec_bytes = 1;            // widest vector all offsets, strides and runs allow (1..16)
  int unroll = 8;               // vectors per thread per tile (1, 2, 4 or 8)
  bool nontemporal = true;      // streaming (non-temporal) loads/stores, always on
  // Destination-major order, for ops whose boxes all go to the same number m > 1 of shards.  Storing a tile to
  // every destination in turn scatters the writes in flight over all destination buffers (measured 5.1-5.4 TB/s
  // for 32 destinations against 6.8 for a plain fill; 3.4-4.4 for 8 destinations of 512 KiB boxes).  Instead the
  // op's tiles, boxes in source order, are taken in chunks of chunk_tiles (16 MiB of source) whatever box they
  // belong to; launch index = (chunk, destination j, tile of the chunk), the tile goes to the j-th destination
  // of its box: what is in flight writes few shards, in long stretches, and a chunk is re-read once per
  // destination from the L2 of the XCD that read it first (tile counts per chunk are multiples of 8, the number
  // of XCDs, so a tile stays on its XCD; loads are ordinary, not streaming, so that the lines stay cached).  A
  // copy microbenchmark reaches 6.4 / 6.5 / 6.8 TB/s for 2-4 / 8 / 32 destinations this way.
  bool dest_major = false;
  uint32_t chunk_tiles = 0;     // a power of two
  uint32_t src_tiles = 0;       // tiles that cover every box once; n_tiles = src_tiles * dm_count
  uint32_t dm_count = 1;        // m when dest_major, else 1
  // A workgroup stores its tile to dm_fanout consecutive destinations of the box's list (the last group of a list may
  // be shorter), so the launch enumerates dm_groups = ceil(m / dm_fanout) groups instead of m destinations:
  // n_tiles = src_tiles * dm_groups.  Measured on MI355X: with 8 destinations, 2 per workgroup halve the
  // re-reads and the workgroup count and run 8-20 % faster than one (5.7 -> 6.2-6.5 TB/s on five attention pairs,
  // the slowest of them 4.7 -> 5.7), 4 slightly less; with 32 destinations one per workgroup is best (5.95, 5.64,
  // 5.47 TB/s for 1, 2, 4).
  uint32_t dm_fanout = 1, dm_groups = 1;
  uint32_t dm_magic = 0, dm_shift = 0;   // division by dm_groups
  // Sibling boxes (destination-major ops).  Where the destination's contiguous rows are made of pieces from several
  // source shards (a gather along the run: 2 KiB from each of four shards per 8 KiB row, say), the tiles of ONE box
  // write pieces that lie a row apart while the rest of those rows waits for another box, and that costs the memory
  // system a tenth of its rate.  Measured with bare kernels, 1 GiB -> 32 x 1 GiB in this order: 6.78 TB/s for a plain
  // copy, 6.05 for tiles of 2 x 2 KiB lying 8 KiB apart, box after box (the descriptor-driven kernel ran at 5.96 on
  // that pattern: the pattern was its whole deficit), 6.78 again when consecutive tiles take the four column blocks
  // of the same two rows.  So sibling boxes -- same shape, same outer ranges, runs adjacent in the destination -- stand
  // next to each other in the box array, sib_count of them per group, and the kernel lets their tiles alternate:
  // tile t of a group is tile t / sib_count of its box t % sib_count.  Nothing else changes: the scalar loads per
  // wave stay what they were (reading the siblings inside one tile, each wave its own, or through a table of
  // sources beside the boxes, took 6 to 9 scalar loads more per wave -- 17 before -- and the kernel from 5.9 to
  // 4.0-4.9 TB/s: at one vector per lane it is the scalar loads that bound it).
  // Ordinary-order ops alternate in the same way, and there the mirror image counts as well: boxes that read
  // adjacent column blocks of the same source rows for different destinations (a scatter along the run: 16 KiB
  // source rows dealt out in 2 KiB pieces to 8 shards).  Bare kernels, 64 MiB -> 64 MiB of that pattern: plain copy
  // 5.95 TB/s; box after box, destination-major 5.52; boxes in source order without alternation 5.04; consecutive
  // tiles taking the 8 column blocks of the same two source rows 5.83.
  // Runs longer than a tile is wide (then a power of two of column blocks each) alternate run by run: the
  // 2^sib_inner_log2 tiles of a run stay together.
  uint32_t sib_count = 1, sib_magic = 0, sib_shift = 0, sib_inner_log2 = 0;
  bool sib_resorted = false;    // (builder's note to itself: the boxes were put in source order for siblings)
  int tc = 1, tr = 1;           // tile = tc vectors wide (the longest run, at most 256*unroll), tr = 256*unroll / tc rows high
  uint32_t tc_magic = 0, tc_shift = 0;  // division by tc
  uint32_t tiles_per_box = 0;   // > 0 when every box has the same number of tiles
  uint32_t tpb_magic = 0;       // division by tiles_per_box (same scheme as DevBox::magic)
  uint32_t tpb_shift = 0;
  uint32_t n_tiles = 0;
  uint32_t max_grid = 16777215u;  // workgroups per launch (the runtime refuses 2^32 threads and more per grid dimension);
                                // an op with more tiles takes several launches
  std::vector<DevBox> boxes;
  std::vector<int32_t> dst_list;
  int64_t bytes_read = 0, bytes_written = 0;
};

constexpr int kMaxUnroll = 8;

// What a caller may choose about how a plan is lowered to launches (the public redist_options, field for field).
// The defaults are the measured choices; the other settings exist for A/B measurements and for tests that must reach
// a code path on a small problem.  They are part of a plan's identity (the plan cache keys on them).
struct BuildOptions {
  bool merge_runs = true;      // a run of dynslices / of allgathers is one launch; dynslices share the next launch
  bool fold_permute = true;    // the allpermute shares the launch of the alltoall before it (or of the allgathers after it)
  bool lds_staging = true;     // LDS-staged bodies for steps on the contiguous dimension
  bool span_form = true;       // ... and their span form
  bool row_dst_order = true;   // ... and their boxes cut and sorted by destination address
  bool dest_major = true;      // destination-major order for large replicating ops
  int64_t dest_major_min_bytes = 32ll << 20;   // smallest op that takes it; 0 also drops the piece / stretch size conditions
  int unroll = 0;              // vectors per thread of the generic body: 0 = by run length, else 1, 2, 4 or 8
  uint32_t max_grid = 16777215u;   // workgroups per launch: 2^32 threads per grid dimension / 256 threads, minus one
  int dm_fanout = 0;           // destinations a workgroup of the generic destination-major body stores to: 0 = by their
                               // number (2 up to 8 destinations, else 1), else 1 or 2
  // Runs of sibling boxes are shorter than this (bytes).  Measured, 256 MiB dealt from / to 8 shards, alternation off
  // -> on: pieces of the destination's rows +3-5 % at 2-32 KiB runs and +10 % at 64 KiB (1 MiB runs, four a row, in
  // the 32-shard activation reshard: +5 %); pieces of the source's rows +0.5-3 % at 2 KiB and -3 to -7 % from 4 KiB
  // on, so those alternate below 4 KiB only.
  int64_t sib_max_run = 2 << 20;
  bool siblings = true;        // destination-major ops: tiles of boxes whose runs are adjacent pieces of the destination's rows alternate
  int cell_form = 1;           // cell-staged body: 0 never, 1 where the other bodies' stretches are short, 2 wherever
                               // a step qualifies
};

// Build the copy op that takes the device table (shape_s, offs_s) to (shape_d, offs_d).
// Returns false if the op exceeds the executor's limits (rows or tiles beyond 2^31).
// Reciprocal for exact division of n < 2^31 by d > 1: n / d == umulhi(n, magic) >> shift.
void magic_for(uint32_t d, uint32_t* magic, uint8_t* shift);

bool build_copy_op(int kind, int ndev, int rank, int elem_size, const std::vector<int64_t>& shape_s,
                   const std::vector<int64_t>& offs_s, const std::vector<int64_t>& shape_d,
                   const std::vector<int64_t>& offs_d, const BuildOptions& opt, CopyOp* out);

// Row-complete description of the same step; returns false when the step does not qualify (last
// dimension untouched, runs long enough for the generic kernel, sizes not powers of two, ...).
bool build_row_op(int ndev, int rank, int elem_size, const std::vector<int64_t>& shape_s,
                  const std::vector<int64_t>& offs_s, const std::vector<int64_t>& shape_d,
                  const std::vector<int64_t>& offs_d, const BuildOptions& opt, RowOp* out);

// Dims at the end of both tile shapes with equal extents are not touched by the step: each is folded into the dim
// before it, and which of its tiles a device holds becomes a new leading dim of extent 1 (no shard's memory layout
// changes).  Returns false when nothing but untouched dims is left.
bool fold_untouched_last_dims(int ndev, int rank, std::vector<int64_t>* shape_s, std::vector<int64_t>* offs_s,
                              std::vector<int64_t>* shape_d, std::vector<int64_t>* offs_d);

// What build_cell_op is told about the body that would otherwise carry out the step.
struct OtherBody {
  int64_t stretch = 0;       // shortest stretch it reads or writes per shard and tile, bytes
  bool strong = true;        // it moves 16-byte vectors on both sides
  bool dest_major = false;   // it runs in destination-major order
};
// Cell-complete description of the same step (see DevCellBox).  Returns false when the step does not qualify or the
// other body is expected to be as good.
bool build_cell_op(int ndev, int rank, int elem_size, const std::vector<int64_t>& shape_s,
                   const std::vector<int64_t>& offs_s, const std::vector<int64_t>& shape_d,
                   const std::vector<int64_t>& offs_d, const BuildOptions& opt, const OtherBody& other, CellOp* out);

}  // namespace redist
