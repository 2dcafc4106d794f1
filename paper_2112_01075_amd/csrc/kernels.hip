// gfx950 kernels: every redistribution step is an index-mapped, HBM-bound copy of boxes between
// shard buffers.  One launch covers all shards of the virtual mesh.
//
// Work decomposition: a box (a strided r-dimensional piece of one source shard that lands in one
// or several destination shards) is cut into tiles of up to 256*kUnroll vectors, tc vectors wide
// along the contiguous run.  A workgroup of 256 threads (4 wavefronts of 64) copies one tile:
// block-uniform values (box, tile position, base pointers) are derived from blockIdx once and sit
// in scalar registers; each lane issues kUnroll independent 16-byte loads before its stores, and
// a row's offsets come from multiply-high divisions by precomputed reciprocals.  A box that
// several shards receive (allgather, replicated targets) is read once and stored to each -- or, for
// large ops, in destination-major order: one workgroup per (tile, receiving shard), 16 MiB of source at
// a time, re-read from the L2.  Steps that split or merge the contiguous dimension into short pieces
// go through LDS instead (row_tile and its general and span forms below), so that both sides see long
// contiguous stretches.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <type_traits>

#include "copyop.hpp"
#include "launch.hpp"

namespace redist {

template <int V> struct VecOf;
template <> struct VecOf<16> { typedef unsigned int type __attribute__((ext_vector_type(4))); };
template <> struct VecOf<8> { typedef unsigned int type __attribute__((ext_vector_type(2))); };
template <> struct VecOf<4> { typedef unsigned int type; };
template <> struct VecOf<2> { typedef unsigned short type; };
template <> struct VecOf<1> { typedef unsigned char type; };

// What a workgroup of the destination-major body needs from the kernel arguments, as two 64-byte vectors: a wave
// fetches them with two scalar loads and one wait instead of a dozen loads and three waits.  (At one vector per lane
// the scalar loads in front of a wave's only vector load are what bounds these kernels: measured on the 32-shard
// gather, six scalar loads more per wave -- 17 before -- cost 22 % of its rate.)
typedef uint32_t u32x16 __attribute__((ext_vector_type(16)));
struct alignas(64) DmHot { u32x16 v[2]; };
enum : int {   // v[0]
  kH_n_tiles = 0, kH_tile_base, kH_chunk_tiles, kH_src_tiles, kH_dm_count, kH_dm_magic, kH_dm_shift, kH_dm_dests,
  kH_tiles_per_box, kH_tpb_magic, kH_tpb_shift, kH_n_boxes, kH_tc, kH_tr, kH_tc_magic, kH_tc_shift
};
enum : int {   // v[1]
  kG_n_outer = 0, kG_common_first, kG_sib_count, kG_sib_magic, kG_sib_shift, kG_sib_group_tiles, kG_sib_gt_magic,
  kG_sib_gt_shift, kG_boxes_lo, kG_boxes_hi, kG_list_lo, kG_list_hi, kG_ss0_lo, kG_ss0_hi, kG_ds0_lo, kG_ds0_hi
};

struct OpArgs {
  const DevBox* __restrict__ boxes;
  const int32_t* __restrict__ dst_list;
  int64_t sstride[kMaxOuter];
  int64_t dstride[kMaxOuter];
  uint32_t n_boxes;
  uint32_t n_tiles;
  uint32_t tiles_per_box;
  uint32_t tpb_magic, tpb_shift;
  int32_t n_outer;
  uint32_t tc, tr, tc_magic, tc_shift;
  uint32_t chunk_tiles;   // destination-major order: tiles per chunk,
  uint32_t src_tiles;     //   tiles that cover every box once (n_tiles = src_tiles * dm_count),
  uint32_t dm_count, dm_magic, dm_shift;   //   destinations per box and the division by their number
  int32_t dm_common_first;   //   >= 0: every box has this dst_first (one destination list for the whole op)
  uint32_t tile_base;     // launch index of this launch's first workgroup (an op beyond the grid limit takes several launches)
  uint32_t dm_dests;      // destination-major order with several destinations per workgroup: destinations per box (then
                          // dm_count, dm_magic and dm_shift above count and divide by the GROUPS of destinations)
  // Sibling boxes (see CopyOp::sib_count): boxes come in groups of sib_count consecutive boxes of one shape
  // (tiles_per_box tiles each) whose tiles alternate: tile t of a group is tile t / sib_count of its box t % sib_count.
  // sib_magic / sib_shift (bits 0-7) divide by sib_count, sib_gt_magic / sib_gt_shift by the tiles of a group;
  // bits 8 and up of sib_shift: log2 of the tiles of a run that stay together.
  uint32_t sib_count, sib_magic, sib_shift, sib_group_tiles, sib_gt_magic, sib_gt_shift;
  DmHot hot;   // the destination-major body reads these copies (filled in by launch_pt)
};

// Every pointer that reaches these two helpers is device memory.  Saying so (address space 1) matters for
// pointers that were staged in LDS: the compiler cannot trace them back to a kernel argument and would use
// FLAT instructions, whose completion it can only await all at once.
#define REDIST_GLOBAL __attribute__((address_space(1)))
template <int V, bool NT>
__device__ __forceinline__ typename VecOf<V>::type load_vec(const char* p) {
  typedef typename VecOf<V>::type vec_t;
  const REDIST_GLOBAL vec_t* g = (const REDIST_GLOBAL vec_t*)(uintptr_t)p;
  if (NT) return __builtin_nontemporal_load(g);
  return *g;
}
template <int V, bool NT>
__device__ __forceinline__ void store_vec(char* p, typename VecOf<V>::type v) {
  typedef typename VecOf<V>::type vec_t;
  REDIST_GLOBAL vec_t* g = (REDIST_GLOBAL vec_t*)(uintptr_t)p;
  if (NT) __builtin_nontemporal_store(v, g);
  else *g = v;
}

// shift[k] of a box, read as part of its 32-bit word: the hardware has no scalar byte loads, so a plain byte access
// becomes a vector load (with a wait of its own) in the middle of the block-uniform address arithmetic.
template <class BoxRef>
__device__ __forceinline__ uint32_t shift_of(const BoxRef& bx, int k) {
  const auto* words = reinterpret_cast<decltype(&bx.tile_first)>(&bx.shift[0]);   // same address space as the box
  return (words[k >> 2] >> (8 * (k & 3))) & 255u;
}

// kSib: the tiles (1) or the runs of several tiles (2) of sibling boxes alternate (see OpArgs).
template <int V, int kUnroll, bool NT, class PS, class PD, int kSib = 0>
__device__ __forceinline__ void gather_tile(const OpArgs& a, const PS& src, const PD& dst) {
  typedef typename VecOf<V>::type vec_t;
  const uint32_t tile = blockIdx.x + a.tile_base;
  if (tile >= a.n_tiles) return;

  // ---- which box (block-uniform) ----
  uint32_t b, sib_t = 0;
  if (kSib) {
    // consecutive tiles take the sibling boxes of a group in turn (boxes of one shape: no descriptor needed)
    const uint32_t g = __umulhi(tile, a.sib_gt_magic) >> a.sib_gt_shift;
    const uint32_t tig = tile - g * a.sib_group_tiles;
    const uint32_t lg = kSib == 2 ? a.sib_shift >> 8 : 0u, q = tig >> lg;   // (runs of 2^lg tiles stay together)
    const uint32_t o = __umulhi(q, a.sib_magic) >> (a.sib_shift & 31u);
    sib_t = (o << lg) | (tig & ((1u << lg) - 1u));
    b = g * a.sib_count + (q - o * a.sib_count);
  } else if (a.tiles_per_box) {
    b = a.tiles_per_box == 1u ? tile : (__umulhi(tile, a.tpb_magic) >> a.tpb_shift);
  } else {
    uint32_t lo = 0, hi = a.n_boxes - 1;  // last box whose tile_first <= tile
    while (lo < hi) {
      uint32_t mid = (lo + hi + 1) >> 1;
      if (a.boxes[mid].tile_first <= tile) lo = mid; else hi = mid - 1;
    }
    b = lo;
  }
  const DevBox& bx = a.boxes[b];
  const uint32_t t_in_box = kSib ? sib_t : tile - bx.tile_first;
  // (a plain division: with the box's reciprocal instead, or skipped when col_blocks is 1, the compiler places the
  //  descriptor loads of this prologue differently and the body measured 5 % slower on 2 KiB runs)
  const uint32_t rb = t_in_box / bx.col_blocks;
  const uint32_t cb = t_in_box - rb * bx.col_blocks;
  const uint32_t tc = a.tc, tr = a.tr;
  const uint32_t row0 = rb * tr, col0 = cb * tc;
  const uint32_t rows = bx.rows, run_vecs = bx.run_vecs;
  const int n_outer = a.n_outer;

  const char* sbase = static_cast<const char*>(src.at(bx.src_dev)) + bx.src_off;

  // A tile that lies wholly inside its box (the common case) needs no per-lane predicate.
  const bool full = (row0 + tr <= rows) && (col0 + tc <= run_vecs) && (tc * tr == 256u * kUnroll);

  vec_t val[kUnroll];
  int64_t doff[kUnroll];
  bool live[kUnroll];
  // all address arithmetic first, then kUnroll independent loads in flight, then the stores
#pragma unroll
  for (int u = 0; u < kUnroll; ++u) {
    const uint32_t e = (uint32_t)u * 256u + threadIdx.x;
    const uint32_t er = tc == 1u ? e : (__umulhi(e, a.tc_magic) >> a.tc_shift);  // e / tc
    const uint32_t row = row0 + er;
    const uint32_t col = col0 + (e - er * tc);
    live[u] = full || (er < tr && row < rows && col < run_vecs);
    int64_t so = (int64_t)col * V, dof = (int64_t)col * V;
    uint32_t n = row;
    for (int k = n_outer - 1; k > 0; --k) {
      const uint32_t len = bx.len[k];
      const uint32_t q = len == 1u ? n : (__umulhi(n, bx.magic[k]) >> shift_of(bx, k));
      const uint32_t idx = n - q * len;
      so += (int64_t)idx * a.sstride[k];
      dof += (int64_t)idx * a.dstride[k];
      n = q;
    }
    if (n_outer > 0) {
      so += (int64_t)n * a.sstride[0];
      dof += (int64_t)n * a.dstride[0];
    }
    doff[u] = dof;
    // lanes outside the box read the box's first vector (in bounds) and store nothing
    val[u] = load_vec<V, NT>(sbase + (live[u] ? so : (int64_t)0));
  }
  const int32_t nd = bx.dst_count;
  char* dbase = static_cast<char*>(dst.at(bx.dst_dev0)) + bx.dst_off;  // first (usually only) destination
  for (int32_t k = 0;;) {
    if (full) {
#pragma unroll
      for (int u = 0; u < kUnroll; ++u) store_vec<V, NT>(dbase + doff[u], val[u]);
    } else {
#pragma unroll
      for (int u = 0; u < kUnroll; ++u)
        if (live[u]) store_vec<V, NT>(dbase + doff[u], val[u]);
    }
    if (++k >= nd) break;
    dbase = static_cast<char*>(dst.at(a.dst_list[bx.dst_first + k])) + bx.dst_off;
  }
}


// DM: destination-major order, for ops whose boxes all have m = dm_count > 1 destinations.  The launch has m
// times the tiles that cover the boxes once: launch index = (chunk of chunk_tiles tiles, destination j, tile of
// the chunk), chunks running over the op's tiles whatever box they belong to; the tile is stored to the j-th
// destination of its box, and loads are ordinary (cached) ones, because each chunk is read once per destination.
// Keeps the listed block-uniform values where they are at this point of the program: the compiler then has to
// fetch them (scalar loads from the kernel arguments or from a descriptor) together, with one wait, instead of
// sinking every load to its first use behind a wait of its own -- a chain of eight or more scalar-cache round
// trips in front of a workgroup's first vector load otherwise.
#define REDIST_FETCH_NOW1(x) asm volatile("" : "+s"(x))
#define REDIST_FETCH_NOW4(x, y, z, w) asm volatile("" : "+s"(x), "+s"(y), "+s"(z), "+s"(w))
#define REDIST_KFETCH4 REDIST_FETCH_NOW4
#define REDIST_BFETCH4 REDIST_FETCH_NOW4

// kFan: destinations a workgroup stores its tile to (consecutive entries of the box's list; the last group of a list
// may be shorter).  Measured on MI355X: with 8 destinations, 2 per workgroup halve the re-reads and the workgroup
// count and run 8-20 % faster than 1 (five attention pairs 5.7 -> 6.2-6.5 TB/s, the slowest of all 4.7 -> 5.7), 4
// slightly less; with 32 destinations 1 is best (5.95, 5.64, 5.47 TB/s for 1, 2, 4).  A template parameter, so that
// the one-destination code is exactly what it was: a run-time loop over destinations cost that case 16 %.
// kSib: the tiles (1) or the runs of several tiles (2) of sibling boxes alternate (see OpArgs).  (Two forms: the
// few scalar instructions that runs of several tiles add cost the tile-by-tile form 5 % of its rate.)
template <int V, int kUnroll, bool NT, class PS, class PD, int kFan, int kSib = 0>
__device__ __forceinline__ void gather_tile_dm(const OpArgs& a, const PS& src, const PD& dst) {
  typedef typename VecOf<V>::type vec_t;
  // ---- kernel arguments: two 64-byte scalar loads, one wait ----
  u32x16 h0 = a.hot.v[0], h1 = a.hot.v[1];
  asm volatile("" : "+s"(h0), "+s"(h1));
  const uint32_t tile = blockIdx.x + h0[kH_tile_base];
  const uint32_t n_tiles = h0[kH_n_tiles], tiles_per_box = h0[kH_tiles_per_box], tpb_magic = h0[kH_tpb_magic];
  const uint32_t tpb_shift = h0[kH_tpb_shift], tc = h0[kH_tc], tr = h0[kH_tr], tc_magic = h0[kH_tc_magic];
  const uint32_t tc_shift = h0[kH_tc_shift], n_boxes = h0[kH_n_boxes], chunk_tiles = h0[kH_chunk_tiles];
  const uint32_t src_tiles = h0[kH_src_tiles], dm_count = h0[kH_dm_count], dm_magic = h0[kH_dm_magic];
  const uint32_t dm_shift = h0[kH_dm_shift];
  const int32_t n_outer = (int32_t)h1[kG_n_outer];
  // the descriptors do not change while the kernel runs: constant address space, read with scalar loads
  typedef const __attribute__((address_space(4))) DevBox* box_ptr;
  typedef const __attribute__((address_space(4))) int32_t* list_ptr;
  typedef const __attribute__((address_space(4))) u32x16* wide_ptr;
  const box_ptr boxes = (box_ptr)(uintptr_t)(((uint64_t)h1[kG_boxes_hi] << 32) | h1[kG_boxes_lo]);
  const list_ptr dst_list = (list_ptr)(uintptr_t)(((uint64_t)h1[kG_list_hi] << 32) | h1[kG_list_lo]);
  if (tile >= n_tiles) return;

  // ---- launch index -> (tile of the op, which destination); block-uniform; chunk_tiles is a power of two ----
  uint32_t s_tile, which_dst;
  {
    const uint32_t chunk_log2 = 31u - (uint32_t)__builtin_clz(chunk_tiles);
    const uint32_t t_hi = tile >> chunk_log2;                            // = c * dm_count + which_dst in whole chunks
    // (with several destinations per workgroup there may be one group only, which the reciprocal does not cover)
    const uint32_t c = kFan > 1 && dm_count == 1u ? t_hi : (__umulhi(t_hi, dm_magic) >> dm_shift);   // chunk
    const uint32_t here = min(chunk_tiles, src_tiles - (c << chunk_log2));   // tiles of this chunk
    if (here == chunk_tiles) {
      which_dst = t_hi - c * dm_count;
      s_tile = (c << chunk_log2) + (tile & (chunk_tiles - 1u));
    } else {                                                             // the op's last, partial chunk
      const uint32_t r = tile - c * chunk_tiles * dm_count;
      which_dst = r / here;
      s_tile = (c << chunk_log2) + (r - which_dst * here);
    }
  }
  if (kFan > 1) which_dst *= (uint32_t)kFan;   // group of destinations -> its first destination

  // ---- which box ----
  uint32_t b, sib_t = 0;
  if (kSib) {
    // Consecutive tiles take the sibling boxes of a group in turn, so that workgroups running at the same time fill
    // the same destination rows (boxes of one shape: no descriptor is needed to find the box).
    const uint32_t g = __umulhi(s_tile, h1[kG_sib_gt_magic]) >> h1[kG_sib_gt_shift];
    const uint32_t tig = s_tile - g * h1[kG_sib_group_tiles];
    if (kSib == 2) {
      const uint32_t lg = h1[kG_sib_shift] >> 8, q = tig >> lg;        // (runs of 2^lg tiles stay together)
      const uint32_t o = __umulhi(q, h1[kG_sib_magic]) >> (h1[kG_sib_shift] & 31u);
      sib_t = (o << lg) | (tig & ((1u << lg) - 1u));                    // tile of the sibling
      b = g * h1[kG_sib_count] + (q - o * h1[kG_sib_count]);
    } else {
      sib_t = __umulhi(tig, h1[kG_sib_magic]) >> h1[kG_sib_shift];      // tile of the sibling
      b = g * h1[kG_sib_count] + (tig - sib_t * h1[kG_sib_count]);
    }
  } else if (tiles_per_box) {
    b = tiles_per_box == 1u ? s_tile : (__umulhi(s_tile, tpb_magic) >> tpb_shift);
  } else {
    uint32_t lo = 0, hi = n_boxes - 1;  // last box whose tile_first <= s_tile
    while (lo < hi) {
      uint32_t mid = (lo + hi + 1) >> 1;
      if (boxes[mid].tile_first <= s_tile) lo = mid; else hi = mid - 1;
    }
    b = lo;
  }
  // ---- the box's scalars, all at once ----
  // (when every box has the same destination list -- a fully replicated target -- the shard this workgroup stores
  //  to does not depend on the box: its index is fetched along with the box instead of after it)
  const int32_t common_first = (int32_t)h1[kG_common_first];
  int32_t common_dev = common_first >= 0 ? dst_list[common_first + (int32_t)which_dst] : -1;
  const __attribute__((address_space(4))) DevBox& bx = boxes[b];
  // ---- the box: two 64-byte scalar loads ----
  const wide_ptr bw = (wide_ptr)(uintptr_t)(boxes + b);
  u32x16 b0 = bw[0], b1 = bw[1];
  asm volatile("" : "+s"(b0), "+s"(b1), "+s"(common_dev));
  static_assert(offsetof(DevBox, src_off) == 0 && offsetof(DevBox, dst_off) == 8 && offsetof(DevBox, src_dev) == 16 &&
                    offsetof(DevBox, dst_first) == 20 && offsetof(DevBox, run_vecs) == 28 && offsetof(DevBox, rows) == 32 &&
                    offsetof(DevBox, tile_first) == 36 && offsetof(DevBox, col_blocks) == 40 &&
                    offsetof(DevBox, dst_dev0) == 112 && offsetof(DevBox, cb_magic) == 116 && offsetof(DevBox, cb_shift) == 120,
                "the destination-major body reads DevBox fields by their place in two 64-byte vectors");
  int64_t src_off = (int64_t)(((uint64_t)b0[1] << 32) | b0[0]), dst_off = (int64_t)(((uint64_t)b0[3] << 32) | b0[2]);
  const int32_t src_dev = (int32_t)b0[4], dst_first = (int32_t)b0[5], dst_dev0 = (int32_t)b1[12];
  const uint32_t run_vecs = b0[7], rows = b0[8], tile_first = b0[9], col_blocks = b0[10];
  const uint32_t cb_magic = b1[13], cb_shift = b1[14] & 255u;

  const uint32_t t_in_box = kSib ? sib_t : s_tile - tile_first;
  const uint32_t rb = col_blocks == 1u ? t_in_box : (__umulhi(t_in_box, cb_magic) >> cb_shift);
  const uint32_t cb = t_in_box - rb * col_blocks;
  const uint32_t row0 = rb * tr, col0 = cb * tc;

  // both base pointers before the vector loads are issued, so that no scalar round trip is left between the
  // arrival of the data and its store
  // (the destination's index comes with the box unless destination lists differ between boxes and this is not a
  //  list's first entry: only then does one more scalar load stand in front of the two pointer loads)
  int32_t ddev = common_first >= 0 ? common_dev : dst_dev0;
  if (common_first < 0 && which_dst != 0u) ddev = dst_list[dst_first + (int32_t)which_dst];
  uint64_t sbase_addr = (uint64_t)(uintptr_t)src.at(src_dev), dbase_addr = (uint64_t)(uintptr_t)dst.at(ddev);
  asm volatile("" : "+s"(sbase_addr), "+s"(dbase_addr));
  sbase_addr += (uint64_t)src_off;
  dbase_addr += (uint64_t)dst_off;
  const char* sbase = reinterpret_cast<const char*>((uintptr_t)sbase_addr);

  // A tile that lies wholly inside its box (the common case) needs no per-lane predicate.
  const bool full = (row0 + tr <= rows) && (col0 + tc <= run_vecs) && (tc * tr == 256u * kUnroll);

  vec_t val[kUnroll];
  int64_t doff[kUnroll];
  bool live[kUnroll];
  // all address arithmetic first, then kUnroll independent loads in flight, then the stores
#pragma unroll
  for (int u = 0; u < kUnroll; ++u) {
    const uint32_t e = (uint32_t)u * 256u + threadIdx.x;
    const uint32_t er = tc == 1u ? e : (__umulhi(e, tc_magic) >> tc_shift);  // e / tc
    const uint32_t row = row0 + er;
    const uint32_t col = col0 + (e - er * tc);
    live[u] = full || (er < tr && row < rows && col < run_vecs);
    int64_t so = (int64_t)col * V, dof = (int64_t)col * V;
    uint32_t n = row;
    for (int k = n_outer - 1; k > 0; --k) {
      const uint32_t len = bx.len[k];
      const uint32_t q = len == 1u ? n : (__umulhi(n, bx.magic[k]) >> shift_of(bx, k));
      const uint32_t idx = n - q * len;
      so += (int64_t)idx * a.sstride[k];
      dof += (int64_t)idx * a.dstride[k];
      n = q;
    }
    if (n_outer > 0) {
      so += (int64_t)n * (int64_t)(((uint64_t)h1[kG_ss0_hi] << 32) | h1[kG_ss0_lo]);
      dof += (int64_t)n * (int64_t)(((uint64_t)h1[kG_ds0_hi] << 32) | h1[kG_ds0_lo]);
    }
    doff[u] = dof;
    // lanes outside the box read the box's first vector (in bounds) and store nothing
    val[u] = load_vec<V, false>(sbase + (live[u] ? so : (int64_t)0));   // cached: the chunk is read again per destination
  }
  char* dbase = reinterpret_cast<char*>((uintptr_t)dbase_addr);
  if (full) {
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) store_vec<V, NT>(dbase + doff[u], val[u]);
  } else {
#pragma unroll
    for (int u = 0; u < kUnroll; ++u)
      if (live[u]) store_vec<V, NT>(dbase + doff[u], val[u]);
  }
  if (kFan > 1) {   // the other destinations of this workgroup's group
    const uint32_t dm_dests = h0[kH_dm_dests];
#pragma unroll
    for (int i = 1; i < kFan; ++i) {
      if (which_dst + (uint32_t)i >= dm_dests) break;
      char* db = static_cast<char*>(dst.at(dst_list[(common_first >= 0 ? common_first : dst_first) + (int32_t)which_dst + i])) + dst_off;
      if (full) {
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) store_vec<V, NT>(db + doff[u], val[u]);
      } else {
#pragma unroll
        for (int u = 0; u < kUnroll; ++u)
          if (live[u]) store_vec<V, NT>(db + doff[u], val[u]);
      }
    }
  }
}

// One entry point per collective so that profiles attribute time to the step kind.
// DM: 0 = ordinary order (-1, -2: with sibling boxes alternating by tiles, by runs of several tiles); 1, 2 =
// destination-major order with that many destinations per workgroup; 3, 4 and 5, 6 = the same with sibling boxes.
#define REDIST_KERNEL(name)                                                                 \
  template <int V, int U, bool NT, int DM, class PS, class PD>                              \
  __global__ void __launch_bounds__(256) name(OpArgs a, PS src, PD dst) {                   \
    if constexpr (DM > 4) gather_tile_dm<V, U, NT, PS, PD, DM - 4, 2>(a, src, dst);         \
    else if constexpr (DM > 2) gather_tile_dm<V, U, NT, PS, PD, DM - 2, 1>(a, src, dst);    \
    else if constexpr (DM > 0) gather_tile_dm<V, U, NT, PS, PD, DM>(a, src, dst);           \
    else if constexpr (DM < 0) gather_tile<V, U, NT, PS, PD, -DM>(a, src, dst);             \
    else gather_tile<V, U, NT, PS, PD>(a, src, dst);                                        \
  }

REDIST_KERNEL(redist_dynslice_kernel)
REDIST_KERNEL(redist_allgather_kernel)
REDIST_KERNEL(redist_alltoall_kernel)
REDIST_KERNEL(redist_allpermute_kernel)
REDIST_KERNEL(redist_fused_gather_kernel)


// ---- row-complete ops: LDS-staged transposes for steps that split or merge the last dimension ----
struct RowArgs {
  const DevRowBox* __restrict__ boxes;
  const DevPiece* __restrict__ pieces;
  const int32_t* __restrict__ dev_list;
  int64_t wstride[kMaxOuter];
  int64_t nstride[kMaxOuter];
  uint32_t n_boxes, n_tiles, tiles_per_box, tpb_magic, tpb_shift;
  int32_t n_outer, w_log2, n_log2, r_log2, n_pieces, narrow_count;
  // general form (W or N not a power of two)
  uint32_t n_bytes, pitch, cpn, cpn_magic, cpn_shift, wpr, wpr_magic, wpr_shift;
  // span form
  uint32_t w_bytes, rpt, nbm, nbm_magic, nbm_shift, mct, slot, cbw, cbw_magic, cbw_shift;
  uint32_t rpt_magic, rpt_shift;   // general form: rpt = rows per tile, and division by it
  int32_t chunk_dims;
  int64_t w_shard_bytes, n_shard_bytes;
  // destination-major order: n_tiles = src_tiles * dm_count, where dm_count counts the GROUPS of dm_fanout receiving
  // shards (dm_dests shards in all) and dm_magic / dm_shift divide by it
  uint32_t dm_count, dm_magic, dm_shift, chunk_tiles, src_tiles;
  uint32_t tile_base;     // launch index of this launch's first workgroup
  uint32_t dm_fanout, dm_dests;
};

template <int V> struct Log2Of;
template <> struct Log2Of<16> { static constexpr int value = 4; };
template <> struct Log2Of<8> { static constexpr int value = 3; };
template <> struct Log2Of<4> { static constexpr int value = 2; };
template <> struct Log2Of<2> { static constexpr int value = 1; };
template <> struct Log2Of<1> { static constexpr int value = 0; };

// Byte address in the staging area of column byte `col` of staged row `r`: rows are W bytes apart and
// the 16-byte chunks of a row are XOR-swizzled with the row number, so that lanes walking down a
// column (the narrow-side order) spread over all LDS banks while whole-row accesses stay linear.
__device__ __forceinline__ uint32_t stage_addr(uint32_t r, uint32_t col, uint32_t w_log2) {
  const uint32_t chunk_mask = (1u << (w_log2 - 4u)) - 1u;
  return (r << w_log2) + ((((col >> 4) ^ (r & chunk_mask)) << 4) | (col & 15u));
}

// Destination-major order of the staged bodies: launch index -> (tile of the op, which of the dm_count groups of
// shards that receive it).  Block-uniform; chunk_tiles is a power of two.
template <int DIR>
__device__ __forceinline__ void row_dm_index(const RowArgs& a, uint32_t* tile_io, uint32_t* which_out) {
  uint32_t tile = *tile_io;
  const uint32_t chunk_log2 = 31u - (uint32_t)__builtin_clz(a.chunk_tiles);
  const uint32_t t_hi = tile >> chunk_log2;                              // = c * dm_count + which in whole chunks
  // (one group only is possible with several shards per workgroup; the reciprocal does not cover a divisor of 1)
  const uint32_t c = a.dm_count == 1u ? t_hi : (__umulhi(t_hi, a.dm_magic) >> a.dm_shift);   // chunk
  const uint32_t here = min(a.chunk_tiles, a.src_tiles - (c << chunk_log2));   // tiles of this chunk
  if (here == a.chunk_tiles) {
    *which_out = t_hi - c * a.dm_count;
    uint32_t l = tile & (a.chunk_tiles - 1u);
    // A gather's chunk is P stretches, one per source shard, at equal offsets of shards that lie a power of two
    // apart.  Workgroups go to the 8 XCDs in turn, so with consecutive tiles every XCD would keep every eighth
    // piece of each stretch in its L2, where the stretches then share cache sets and push each other out
    // (measured: the source fetched 2.8 times per launch instead of once, 5.3 TB/s).  Instead XCD x takes the
    // x-th eighth of the chunk's tiles: what it keeps of a stretch is dense (1.0 times, 6.4 TB/s).  Scatters
    // read one dense stretch of one shard either way; the generic body's chunk is dense too and measured 4 %
    // slower in this order.
    if (DIR == 0) l = (l & 7u) * (a.chunk_tiles >> 3) + (l >> 3);
    *tile_io = (c << chunk_log2) + l;
  } else {                                                               // the op's last, partial chunk
    const uint32_t rr = tile - c * a.chunk_tiles * a.dm_count;
    const uint32_t which = rr / here;
    *which_out = which;
    *tile_io = (c << chunk_log2) + (rr - which * here);
  }
}

// RMAX: most rows a tile may hold.  256 (one row per thread in phase 0) fills the 16 KiB staging area for wide rows
// of 64 bytes and more; rows of 16 and 32 bytes take the instantiation with 1024, whose larger offset tables cost
// occupancy that only it pays.
// DM: destination-major order.  The launch has dm_count times the tiles of the op: launch index = (chunk of
// chunk_tiles tiles, which of the dm_count shards that receive a tile, tile of the chunk); a workgroup stages its
// tile like any other but stores it to that one shard only, and its loads are ordinary (cached) ones, because the
// chunk is read again for the next shard.
template <int VN, int DIR, class PT, int RMAX = 256, bool DM = false>
__device__ __forceinline__ void row_tile(const RowArgs& a, const PT& src, const PT& dst) {
  typedef typename VecOf<VN>::type vecn_t;
  typedef VecOf<16>::type vecw_t;
  __shared__ __align__(16) unsigned char stage[kRowTileBytes];
  __shared__ int64_t s_woff[RMAX];
  __shared__ int64_t s_noff[RMAX];
  __shared__ char* s_nptr[kRowMaxPtrs];

  uint32_t tile = blockIdx.x + a.tile_base;
  if (tile >= a.n_tiles) return;
  uint32_t which = 0;   // DM: the one shard this workgroup stores to
  if (DM) row_dm_index<DIR>(a, &tile, &which);
  uint32_t b;
  if (a.tiles_per_box) {
    b = a.tiles_per_box == 1u ? tile : (__umulhi(tile, a.tpb_magic) >> a.tpb_shift);
  } else {
    uint32_t lo = 0, hi = a.n_boxes - 1;
    while (lo < hi) {
      uint32_t mid = (lo + hi + 1) >> 1;
      if (a.boxes[mid].tile_first <= tile) lo = mid; else hi = mid - 1;
    }
    b = lo;
  }
  const DevRowBox& bx = a.boxes[b];
  const uint32_t r_log2 = (uint32_t)a.r_log2, w_log2 = (uint32_t)a.w_log2, n_log2 = (uint32_t)a.n_log2;
  const uint32_t R = 1u << r_log2;
  const uint32_t row0 = (tile - bx.tile_first) << r_log2;
  const uint32_t rows_here = min(R, bx.rows - row0);
  const uint32_t tid = threadIdx.x;
  const PT& ntab = DIR == 0 ? src : dst;  // narrow-side shards
  const PT& wtab = DIR == 0 ? dst : src;  // wide-side shards
  const int n_outer = a.n_outer;
  const uint32_t narrow_count = (uint32_t)a.narrow_count;

  // ---- phase 0: per-row offsets on both sides, narrow-side base pointers ----
  for (uint32_t rr = tid; rr < rows_here; rr += 256u) {
    uint32_t n = row0 + rr;
    int64_t wo = 0, no = 0;
    for (int k = n_outer - 1; k > 0; --k) {
      const uint32_t len = bx.len[k];
      const uint32_t q = len == 1u ? n : (__umulhi(n, bx.magic[k]) >> shift_of(bx, k));
      const uint32_t idx = n - q * len;
      wo += (int64_t)idx * a.wstride[k];
      no += (int64_t)idx * a.nstride[k];
      n = q;
    }
    if (n_outer > 0) {
      wo += (int64_t)n * a.wstride[0];
      no += (int64_t)n * a.nstride[0];
    }
    s_woff[rr] = wo;
    s_noff[rr] = no;
  }
  for (uint32_t i = tid; i < (uint32_t)a.n_pieces * narrow_count; i += 256u) {
    const uint32_t k = i / narrow_count, j = i - k * narrow_count;
    const DevPiece pc = a.pieces[bx.piece_first + (int32_t)k];
    s_nptr[i] = static_cast<char*>(ntab.at(a.dev_list[pc.dev_first + (int32_t)j])) + pc.narrow_off;
  }
  // DM: this workgroup's group of receiving shards, [which * dm_fanout, ... + dm_fanout) cut at their number
  const uint32_t g_first = which * a.dm_fanout, g_end = min(g_first + a.dm_fanout, a.dm_dests);
  const uint32_t j_first = DM && DIR == 1 ? g_first : 0u, j_end = DM && DIR == 1 ? g_end : narrow_count;
  const int32_t d_first = DM && DIR == 0 ? (int32_t)g_first : 0, d_end = DM && DIR == 0 ? (int32_t)g_end : bx.wide_count;
  __syncthreads();

  constexpr uint32_t LV = Log2Of<VN>::value;
  const uint32_t cpl = n_log2 - LV;                       // log2(narrow vectors per piece row)
  const uint32_t n_total = (R << w_log2) >> LV;           // narrow vectors per tile (R*W bytes <= 16 KiB)
  const uint32_t wchunks_log2 = w_log2 - 4u;              // log2(16-byte chunks per wide row)

  if (DIR == 0) {
    // ---- gather: narrow-side loads (R consecutive narrow rows are contiguous) -> LDS ----
    for (uint32_t e0 = 0; e0 < n_total; e0 += 1024u) {
      vecn_t v[4];
      uint32_t addr[4];
      bool ok[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const uint32_t e = e0 + (uint32_t)q * 256u + tid;
        const uint32_t c = e & ((1u << cpl) - 1u);
        const uint32_t r = (e >> cpl) & (R - 1u);
        const uint32_t k = e >> (cpl + r_log2);
        ok[q] = e < n_total && r < rows_here;
        addr[q] = stage_addr(r, (k << n_log2) + (c << LV), w_log2);
        const char* p = ok[q] ? s_nptr[k] + s_noff[r] + ((int64_t)c << LV) : s_nptr[0];
        v[q] = load_vec<VN, !DM>(p);
      }
#pragma unroll
      for (int q = 0; q < 4; ++q)
        if (ok[q]) *reinterpret_cast<vecn_t*>(stage + addr[q]) = v[q];
    }
    __syncthreads();
    // ---- whole wide rows LDS -> every destination shard of the box ----
    vecw_t v[4];
    int64_t off[4];
    bool ok[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const uint32_t e = (uint32_t)q * 256u + tid;
      const uint32_t w = e & ((1u << wchunks_log2) - 1u);
      const uint32_t r = e >> wchunks_log2;
      ok[q] = r < rows_here;
      v[q] = *reinterpret_cast<const vecw_t*>(stage + stage_addr(r, w << 4, w_log2));
      off[q] = (ok[q] ? s_woff[r] : 0) + ((int64_t)w << 4);
    }
    for (int32_t d = d_first; d < d_end; ++d) {
      char* base = static_cast<char*>(wtab.at(a.dev_list[bx.wide_first + d])) + bx.wide_off;
#pragma unroll
      for (int q = 0; q < 4; ++q)
        if (ok[q]) store_vec<16, true>(base + off[q], v[q]);
    }
  } else {
    // ---- scatter: whole wide rows of the first wide-side shard -> LDS ----
    {
      const char* base = static_cast<const char*>(wtab.at(a.dev_list[bx.wide_first])) + bx.wide_off;
      vecw_t v[4];
      uint32_t addr[4];
      bool ok[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const uint32_t e = (uint32_t)q * 256u + tid;
        const uint32_t w = e & ((1u << wchunks_log2) - 1u);
        const uint32_t r = e >> wchunks_log2;
        ok[q] = r < rows_here;
        addr[q] = stage_addr(r, w << 4, w_log2);
        v[q] = load_vec<16, !DM>(base + (ok[q] ? s_woff[r] + ((int64_t)w << 4) : (int64_t)0));
      }
#pragma unroll
      for (int q = 0; q < 4; ++q)
        if (ok[q]) *reinterpret_cast<vecw_t*>(stage + addr[q]) = v[q];
    }
    __syncthreads();
    // ---- LDS -> narrow side: piece k of R consecutive rows is one contiguous stretch per shard ----
    if (cpl == 0u) {
      // One vector per piece row (pieces of 4 to 16 bytes): a thread keeps its row and walks the pieces, so the
      // row's offset is fetched once and the index arithmetic per vector shrinks to the piece number.  Measured on
      // 4-byte pieces: 30 vector-ALU instructions per vector in the general loop below, the kernel 44 % ALU-busy;
      // this loop gains 6-7 % there.  (The same loop on the load side of a gather has too few loads in flight with
      // two pieces per row: measured 12-22 % slower, so gathers keep the general loop.)
      const uint32_t rl = min(r_log2, 8u), kstep = 256u >> rl, k0 = tid >> rl, np = (uint32_t)a.n_pieces;
      for (uint32_t rb = 0; rb < R; rb += 256u) {
        const uint32_t r = rb + (tid & ((1u << rl) - 1u));
        if (r < rows_here) {
          const int64_t o = s_noff[r];
#pragma unroll 4
          for (uint32_t k = k0; k < np; k += kstep) {
            const vecn_t v = *reinterpret_cast<const vecn_t*>(stage + stage_addr(r, k << n_log2, w_log2));
            for (uint32_t j = j_first; j < j_end; ++j) store_vec<VN, true>(s_nptr[k * narrow_count + j] + o, v);
          }
        }
      }
    } else
    for (uint32_t e0 = 0; e0 < n_total; e0 += 1024u) {
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const uint32_t e = e0 + (uint32_t)q * 256u + tid;
        const uint32_t c = e & ((1u << cpl) - 1u);
        const uint32_t r = (e >> cpl) & (R - 1u);
        const uint32_t k = e >> (cpl + r_log2);
        if (e < n_total && r < rows_here) {
          const vecn_t v = *reinterpret_cast<const vecn_t*>(stage + stage_addr(r, (k << n_log2) + (c << LV), w_log2));
          const int64_t o = s_noff[r] + ((int64_t)c << LV);
          for (uint32_t j = j_first; j < j_end; ++j) store_vec<VN, true>(s_nptr[k * narrow_count + j] + o, v);
        }
      }
    }
  }
}


// General form of the row-complete body: W and N need not be powers of two.  Both sides move vectors
// of V bytes; staged rows are `pitch` bytes apart; indices come from reciprocal divisions.
template <int VW, int V, int DIR, class PT, bool DM = false>
__device__ __forceinline__ void row_tile_general(const RowArgs& a, const PT& src, const PT& dst) {
  typedef typename VecOf<V>::type vec_t;     // narrow side
  typedef typename VecOf<VW>::type vecw_t;   // wide side (16 bytes when rows and offsets allow, else V)
  __shared__ __align__(16) unsigned char stage[kRowTileBytes];
  __shared__ int64_t s_woff[256];
  __shared__ int64_t s_noff[256];
  __shared__ char* s_nptr[kRowMaxPtrs];

  uint32_t tile = blockIdx.x + a.tile_base;
  if (tile >= a.n_tiles) return;
  uint32_t which = 0;   // DM: the one shard this workgroup stores to
  if (DM) row_dm_index<DIR>(a, &tile, &which);
  uint32_t b;
  if (a.tiles_per_box) {
    b = a.tiles_per_box == 1u ? tile : (__umulhi(tile, a.tpb_magic) >> a.tpb_shift);
  } else {
    uint32_t lo = 0, hi = a.n_boxes - 1;
    while (lo < hi) {
      uint32_t mid = (lo + hi + 1) >> 1;
      if (a.boxes[mid].tile_first <= tile) lo = mid; else hi = mid - 1;
    }
    b = lo;
  }
  const DevRowBox& bx = a.boxes[b];
  const uint32_t R = a.rpt;   // rows per tile: any number up to 256
  const uint32_t row0 = (tile - bx.tile_first) * R;
  const uint32_t rows_here = min(R, bx.rows - row0);
  const uint32_t tid = threadIdx.x;
  const PT& ntab = DIR == 0 ? src : dst;
  const PT& wtab = DIR == 0 ? dst : src;
  const int n_outer = a.n_outer;
  const uint32_t narrow_count = (uint32_t)a.narrow_count;

  if (tid < rows_here) {
    uint32_t n = row0 + tid;
    int64_t wo = 0, no = 0;
    for (int k = n_outer - 1; k > 0; --k) {
      const uint32_t len = bx.len[k];
      const uint32_t q = len == 1u ? n : (__umulhi(n, bx.magic[k]) >> shift_of(bx, k));
      const uint32_t idx = n - q * len;
      wo += (int64_t)idx * a.wstride[k];
      no += (int64_t)idx * a.nstride[k];
      n = q;
    }
    if (n_outer > 0) {
      wo += (int64_t)n * a.wstride[0];
      no += (int64_t)n * a.nstride[0];
    }
    s_woff[tid] = wo;
    s_noff[tid] = no;
  }
  for (uint32_t i = tid; i < (uint32_t)a.n_pieces * narrow_count; i += 256u) {
    const uint32_t k = i / narrow_count, j = i - k * narrow_count;
    const DevPiece pc = a.pieces[bx.piece_first + (int32_t)k];
    s_nptr[i] = static_cast<char*>(ntab.at(a.dev_list[pc.dev_first + (int32_t)j])) + pc.narrow_off;
  }
  const uint32_t g_first = which * a.dm_fanout, g_end = min(g_first + a.dm_fanout, a.dm_dests);
  const uint32_t j_first = DM && DIR == 1 ? g_first : 0u, j_end = DM && DIR == 1 ? g_end : narrow_count;
  const int32_t d_first = DM && DIR == 0 ? (int32_t)g_first : 0, d_end = DM && DIR == 0 ? (int32_t)g_end : bx.wide_count;
  __syncthreads();

  const uint32_t n_total = R * (uint32_t)a.n_pieces * a.cpn;  // narrow vectors per tile
  const uint32_t w_total = R * a.wpr;                          // wide vectors per tile
  const uint32_t pitch = a.pitch, cpn = a.cpn, wpr = a.wpr, n_bytes = a.n_bytes;

  // narrow-side element e: vector c of piece k in staged row r (c fastest, then r, then k)
#define REDIST_NARROW_INDEX(e, c, r, k)                                                      \
  const uint32_t t_##e = cpn == 1u ? (e) : (__umulhi((e), a.cpn_magic) >> a.cpn_shift);      \
  const uint32_t c = (e) - t_##e * cpn;                                                      \
  const uint32_t k = __umulhi(t_##e, a.rpt_magic) >> a.rpt_shift;                            \
  const uint32_t r = t_##e - k * R;
  // wide-side element e: vector w of staged row r
#define REDIST_WIDE_INDEX(e, w, r)                                                           \
  const uint32_t r = wpr == 1u ? (e) : (__umulhi((e), a.wpr_magic) >> a.wpr_shift);          \
  const uint32_t w = (e) - r * wpr;

  if (DIR == 0) {
    for (uint32_t e0 = 0; e0 < n_total; e0 += 1024u) {
      vec_t v[4];
      uint32_t addr[4];
      bool ok[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const uint32_t e = e0 + (uint32_t)q * 256u + tid;
        REDIST_NARROW_INDEX(e, c, r, k)
        ok[q] = e < n_total && r < rows_here;
        addr[q] = r * pitch + k * n_bytes + c * (uint32_t)V;
        const char* p = ok[q] ? s_nptr[k] + s_noff[r] + (int64_t)(c * (uint32_t)V) : s_nptr[0];
        v[q] = load_vec<V, !DM>(p);
      }
#pragma unroll
      for (int q = 0; q < 4; ++q)
        if (ok[q]) *reinterpret_cast<vec_t*>(stage + addr[q]) = v[q];
    }
    __syncthreads();
    for (uint32_t e0 = 0; e0 < w_total; e0 += 1024u) {
      vecw_t v[4];
      int64_t off[4];
      bool ok[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const uint32_t e = e0 + (uint32_t)q * 256u + tid;
        REDIST_WIDE_INDEX(e, w, r)
        ok[q] = e < w_total && r < rows_here;
        if (ok[q]) {
          v[q] = *reinterpret_cast<const vecw_t*>(stage + r * pitch + w * (uint32_t)VW);
          off[q] = s_woff[r] + (int64_t)(w * (uint32_t)VW);
        }
      }
      for (int32_t d = d_first; d < d_end; ++d) {
        char* base = static_cast<char*>(wtab.at(a.dev_list[bx.wide_first + d])) + bx.wide_off;
#pragma unroll
        for (int q = 0; q < 4; ++q)
          if (ok[q]) store_vec<VW, true>(base + off[q], v[q]);
      }
    }
  } else {
    const char* base = static_cast<const char*>(wtab.at(a.dev_list[bx.wide_first])) + bx.wide_off;
    for (uint32_t e0 = 0; e0 < w_total; e0 += 1024u) {
      vecw_t v[4];
      uint32_t addr[4];
      bool ok[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const uint32_t e = e0 + (uint32_t)q * 256u + tid;
        REDIST_WIDE_INDEX(e, w, r)
        ok[q] = e < w_total && r < rows_here;
        addr[q] = r * pitch + w * (uint32_t)VW;
        v[q] = load_vec<VW, !DM>(base + (ok[q] ? s_woff[r] + (int64_t)(w * (uint32_t)VW) : (int64_t)0));
      }
#pragma unroll
      for (int q = 0; q < 4; ++q)
        if (ok[q]) *reinterpret_cast<vecw_t*>(stage + addr[q]) = v[q];
    }
    __syncthreads();
    for (uint32_t e0 = 0; e0 < n_total; e0 += 1024u) {
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const uint32_t e = e0 + (uint32_t)q * 256u + tid;
        REDIST_NARROW_INDEX(e, c, r, k)
        if (e < n_total && r < rows_here) {
          const vec_t v = *reinterpret_cast<const vec_t*>(stage + r * pitch + k * n_bytes + c * (uint32_t)V);
          const int64_t o = s_noff[r] + (int64_t)(c * (uint32_t)V);
          for (uint32_t j = j_first; j < j_end; ++j) store_vec<V, true>(s_nptr[k * narrow_count + j] + o, v);
        }
      }
    }
  }
#undef REDIST_NARROW_INDEX
#undef REDIST_WIDE_INDEX
}

// Span form of the row-complete body, for rows that start at odd multiples of a granule of G < 16 bytes.
// Rows that are contiguous on both sides form chunks; a tile is up to mct virtual chunks (whole chunks, or
// stretches of rpt rows of a long one), each of them one contiguous span per side: rows*W bytes on the wide
// side, rows*N bytes per piece on the narrow side.  Each span is covered by 16-byte ALIGNED blocks of
// global memory.  The staging area gives every virtual chunk `slot` bytes and holds it in the wide side's
// byte order, shifted by the wide span's misalignment, so that a wide block is one aligned 16-byte LDS
// access; narrow blocks are taken apart into granules, each with its own (row, column) in the staging area.
//   loads : a block is read whole even when only part of it belongs to the span (the rest is dropped), as
//           long as it lies inside the shard: no block but the very last of a shard whose size is not a
//           multiple of 16 fails that, and that one is read granule by granule.  Every lane issues its
//           loads unconditionally (a branch around a load makes the compiler await each load in turn);
//           lanes without a block read the tile's first block instead.
//   stores: whole blocks as vectors; the first and last block of a span only where they belong to it,
//           granule by granule (their other bytes belong to neighbouring tiles).
// Geometry of virtual chunk v of a box: offsets of its first row on both sides, and its row count.
__device__ __forceinline__ void span_chunk_geometry(const RowArgs& a, const DevRowBox& bx, uint32_t v, int64_t* wo_out,
                                                    int64_t* no_out, uint32_t* rows_out) {
  const uint32_t o = bx.tpc == 1u ? v : (__umulhi(v, bx.tpc_magic) >> bx.tpc_shift);   // chunk; v - o*tpc = stretch in it
  const uint32_t r0 = (v - o * bx.tpc) * bx.vrows;
  *rows_out = min(bx.vrows, bx.chunk_rows - r0);
  int64_t wo = (int64_t)r0 * a.w_bytes, no = (int64_t)r0 * a.n_bytes;
  uint32_t n = o;
  for (int k = a.chunk_dims - 1; k > 0; --k) {
    const uint32_t len = bx.len[k];
    const uint32_t q = len == 1u ? n : (__umulhi(n, bx.magic[k]) >> shift_of(bx, k));
    const uint32_t idx = n - q * len;
    wo += (int64_t)idx * a.wstride[k];
    no += (int64_t)idx * a.nstride[k];
    n = q;
  }
  if (a.chunk_dims > 0) {
    wo += (int64_t)n * a.wstride[0];
    no += (int64_t)n * a.nstride[0];
  }
  *wo_out = wo;
  *no_out = no;
}

template <int G, int DIR, class PT, bool DM = false>
__device__ __forceinline__ void row_tile_span(const RowArgs& a, const PT& src, const PT& dst) {
  typedef typename VecOf<G>::type gran_t;
  typedef VecOf<16>::type vec16;
  constexpr int GP = 16 / G;  // granules per block
  union Block { vec16 v; gran_t g[GP]; };
  __shared__ __align__(16) unsigned char stage[kRowTileBytes + 32];
  // per (virtual chunk, piece): the narrow span rounded down to 16 bytes, for each narrow-side shard
  __shared__ char* s_nptr[kRowMaxPtrs];
  __shared__ uint32_t s_na[kRowMaxPtrs];   // what the rounding took off | span bytes << 4
  __shared__ uint32_t s_nb[kRowMaxPtrs];   // staging address of the span's first byte | blocks to the shard's end << 16
  // per virtual chunk: the wide span
  __shared__ int64_t s_wblk[kRowMaxChunks];  // offset in the wide shard(s), rounded down to 16 bytes
  __shared__ uint32_t s_wa[kRowMaxChunks];   // what the rounding took off | span bytes << 4
  __shared__ uint32_t s_wlim[kRowMaxChunks]; // blocks to the shard's end

  uint32_t tile = blockIdx.x + a.tile_base;
  if (tile >= a.n_tiles) return;
  uint32_t which = 0;   // DM: the one shard this workgroup stores to
  if (DM) row_dm_index<DIR>(a, &tile, &which);
  uint32_t b;
  if (a.tiles_per_box) {
    b = a.tiles_per_box == 1u ? tile : (__umulhi(tile, a.tpb_magic) >> a.tpb_shift);
  } else {
    uint32_t lo = 0, hi = a.n_boxes - 1;
    while (lo < hi) {
      uint32_t mid = (lo + hi + 1) >> 1;
      if (a.boxes[mid].tile_first <= tile) lo = mid; else hi = mid - 1;
    }
    b = lo;
  }
  const DevRowBox& bx = a.boxes[b];
  const uint32_t tid = threadIdx.x;
  const PT& ntab = DIR == 0 ? src : dst;
  const PT& wtab = DIR == 0 ? dst : src;
  const uint32_t narrow_count = (uint32_t)a.narrow_count;
  const uint32_t W = a.w_bytes, N = a.n_bytes, P = (uint32_t)a.n_pieces;
  const uint32_t v0 = (tile - bx.tile_first) * a.mct;          // first virtual chunk of the tile
  const uint32_t m_here = min(a.mct, bx.n_vchunks - v0);

  // ---- where every span of the tile starts ----
  for (uint32_t i = tid; i < m_here * P * narrow_count; i += 256u) {
    const uint32_t vk = i / narrow_count, jn = i - vk * narrow_count;
    const uint32_t c = vk / P, k = vk - c * P;
    int64_t wo, no;
    uint32_t rows;
    span_chunk_geometry(a, bx, v0 + c, &wo, &no, &rows);
    const DevPiece pc = a.pieces[bx.piece_first + (int32_t)k];
    const int64_t off = pc.narrow_off + no, blk0 = off & ~(int64_t)15;
    s_nptr[i] = static_cast<char*>(ntab.at(a.dev_list[pc.dev_first + (int32_t)jn])) + blk0;
    if (jn == 0) {
      const uint32_t pw = (uint32_t)((bx.wide_off + wo) & 15);
      const uint32_t lim = (uint32_t)min((a.n_shard_bytes - blk0) >> 4, (int64_t)0xffff);
      s_na[vk] = (uint32_t)(off & 15) | ((rows * N) << 4);
      s_nb[vk] = (c * a.slot + pw + k * N) | (lim << 16);
    }
  }
  if (tid < m_here) {
    int64_t wo, no;
    uint32_t rows;
    span_chunk_geometry(a, bx, v0 + tid, &wo, &no, &rows);
    const int64_t woff = bx.wide_off + wo, blk0 = woff & ~(int64_t)15;
    s_wblk[tid] = blk0;
    s_wa[tid] = (uint32_t)(woff & 15) | ((rows * W) << 4);
    s_wlim[tid] = (uint32_t)min((a.w_shard_bytes - blk0) >> 4, (int64_t)0x7fffffff);
  }
  __syncthreads();

  const uint32_t g_first = which * a.dm_fanout, g_end = min(g_first + a.dm_fanout, a.dm_dests);
  const uint32_t jn_first = DM && DIR == 1 ? g_first : 0u, jn_end = DM && DIR == 1 ? g_end : narrow_count;
  const int32_t d_first = DM && DIR == 0 ? (int32_t)g_first : 0, d_end = DM && DIR == 0 ? (int32_t)g_end : bx.wide_count;
  const uint32_t n_items = m_here * P * a.nbm;   // (virtual chunk, piece, block) triples of the narrow side
  const uint32_t w_items = m_here * a.cbw;       // (virtual chunk, block) pairs of the wide side
  const uint32_t cpn = a.cpn;

  // item e of the narrow side: block j of span vk = (virtual chunk, piece); s0 = span byte of the block's first
  // granule (may be < 0); len = bytes of the span; sb = staging address of the span's first byte
#define REDIST_SPAN_ITEM(e, vk, j, s0, len, sb, lim, any)                                     \
  const uint32_t vk = __umulhi((e), a.nbm_magic) >> a.nbm_shift;                              \
  const uint32_t j = (e) - vk * a.nbm;                                                        \
  const uint32_t na_##vk = (e) < n_items ? s_na[vk] : 0u, nb_##vk = (e) < n_items ? s_nb[vk] : 0u; \
  const int32_t s0 = (int32_t)(j << 4) - (int32_t)(na_##vk & 15u);                            \
  const int32_t len = (int32_t)(na_##vk >> 4);                                                \
  const uint32_t sb = nb_##vk & 0xffffu, lim = nb_##vk >> 16;                                 \
  const bool any = (e) < n_items && s0 < len;
  // item e of the wide side: block j of virtual chunk c
#define REDIST_SPAN_WITEM(e, c, j, s0, len, any)                                              \
  const uint32_t c = a.mct == 1u ? 0u : (__umulhi((e), a.cbw_magic) >> a.cbw_shift);          \
  const uint32_t j = (e) - c * a.cbw;                                                         \
  const uint32_t wa_##c = (e) < w_items ? s_wa[c] : 0u;                                       \
  const int32_t s0 = (int32_t)(j << 4) - (int32_t)(wa_##c & 15u);                             \
  const int32_t len = (int32_t)(wa_##c >> 4);                                                 \
  const bool any = (e) < w_items && s0 < len;
  // Staging address of the block's first granule inside the span (granule g0), and the walk to the next
  // granule: one granule further in the piece row, or on to the next wide row when the piece row ends.
#define REDIST_SPAN_FIRST(s0, sb, g0, ad, col)                                                \
  const int g0 = (s0) < 0 ? (-(s0)) / G : 0;                                                  \
  const uint32_t sg_##ad = (uint32_t)((s0) + g0 * G) / (uint32_t)G;                           \
  const uint32_t row_##ad = cpn == 1u ? sg_##ad : (__umulhi(sg_##ad, a.cpn_magic) >> a.cpn_shift); \
  uint32_t col = sg_##ad - row_##ad * cpn;                                                    \
  uint32_t ad = (sb) + row_##ad * W + col * (uint32_t)G;
#define REDIST_SPAN_NEXT(ad, col)                                                             \
  {                                                                                           \
    ++col;                                                                                    \
    ad += (uint32_t)G;                                                                        \
    if (col == cpn) { col = 0; ad += W - N; }                                                 \
  }

  if (DIR == 0) {
    // ---- gather: narrow spans -> staging area ----
    const bool vec_ok = (s_nb[0] >> 16) > 0u;   // block-uniform: the tile's first block can stand in for lanes without one
    for (uint32_t e0 = 0; e0 < n_items; e0 += 1024u) {
      Block blk[4];
      int32_t s0s[4], lens[4];
      uint32_t vks[4], js[4], sbs[4];
      bool vecs[4], slow[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const uint32_t e = e0 + (uint32_t)q * 256u + tid;
        REDIST_SPAN_ITEM(e, vk, j, s0, len, sb, lim, any)
        const bool vec = any && vec_ok && j < lim;
        s0s[q] = s0; lens[q] = len; vks[q] = vk; js[q] = j; sbs[q] = sb; vecs[q] = vec; slow[q] = any && !vec;
      }
      if (vec_ok) {
#pragma unroll
        for (int q = 0; q < 4; ++q)
          blk[q].v = load_vec<16, !DM>(s_nptr[(vecs[q] ? vks[q] : 0u) * narrow_count] + ((int64_t)(vecs[q] ? js[q] : 0u) << 4));
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          if (!vecs[q]) continue;
          REDIST_SPAN_FIRST(s0s[q], sbs[q], g0, ad, col)
#pragma unroll
          for (int g = 0; g < GP; ++g) {
            if (g < g0) continue;
            if (s0s[q] + g * G < lens[q]) *reinterpret_cast<gran_t*>(stage + ad) = blk[q].g[g];
            REDIST_SPAN_NEXT(ad, col)
          }
        }
      }
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        if (!slow[q]) continue;   // the block that reaches past the end of the shard
        const char* p = s_nptr[vks[q] * narrow_count] + ((int64_t)js[q] << 4);
        REDIST_SPAN_FIRST(s0s[q], sbs[q], g0, ad, col)
        for (int g = g0; g < GP && s0s[q] + g * G < lens[q]; ++g) {
          *reinterpret_cast<gran_t*>(stage + ad) = load_vec<G, false>(p + g * G);
          REDIST_SPAN_NEXT(ad, col)
        }
      }
    }
    __syncthreads();
    // ---- staging area -> wide spans of every wide-side shard ----
    for (uint32_t e0 = 0; e0 < w_items; e0 += 1024u) {
      Block blk[4];
      int32_t s0s[4], lens[4];
      int64_t offs[4];
      bool anys[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const uint32_t e = e0 + (uint32_t)q * 256u + tid;
        REDIST_SPAN_WITEM(e, c, j, s0, len, any)
        s0s[q] = s0; lens[q] = len; anys[q] = any;
        if (any) {
          blk[q].v = *reinterpret_cast<const vec16*>(stage + c * a.slot + (j << 4));
          offs[q] = s_wblk[c] + ((int64_t)j << 4);
        }
      }
      for (int32_t d = d_first; d < d_end; ++d) {
        char* base = static_cast<char*>(wtab.at(a.dev_list[bx.wide_first + d]));
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          if (!anys[q]) continue;
          if (s0s[q] >= 0 && s0s[q] + 16 <= lens[q]) {
            store_vec<16, true>(base + offs[q], blk[q].v);
          } else {
#pragma unroll
            for (int g = 0; g < GP; ++g) {
              const int32_t sb = s0s[q] + g * G;
              if (sb >= 0 && sb < lens[q]) store_vec<G, false>(base + offs[q] + g * G, blk[q].g[g]);
            }
          }
        }
      }
    }
  } else {
    // ---- scatter: wide spans of the first wide-side shard -> staging area ----
    const char* base = static_cast<const char*>(wtab.at(a.dev_list[bx.wide_first]));
    const bool vec_ok = s_wlim[0] > 0u;
    for (uint32_t e0 = 0; e0 < w_items; e0 += 1024u) {
      int32_t s0s[4], lens[4];
      uint32_t ads[4];
      int64_t offs[4];
      bool vecs[4], slow[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const uint32_t e = e0 + (uint32_t)q * 256u + tid;
        REDIST_SPAN_WITEM(e, c, j, s0, len, any)
        const bool vec = any && vec_ok && j < s_wlim[any ? c : 0u];
        s0s[q] = s0; lens[q] = len; vecs[q] = vec; slow[q] = any && !vec;
        ads[q] = c * a.slot + (j << 4);
        offs[q] = vec || slow[q] ? s_wblk[c] + ((int64_t)j << 4) : s_wblk[0];
      }
      if (vec_ok) {
        vec16 v[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) v[q] = load_vec<16, !DM>(base + (vecs[q] ? offs[q] : s_wblk[0]));
#pragma unroll
        for (int q = 0; q < 4; ++q)
          if (vecs[q]) *reinterpret_cast<vec16*>(stage + ads[q]) = v[q];
      }
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        if (!slow[q]) continue;   // the block that reaches past the end of the shard
        for (int g = 0; g < GP; ++g) {
          const int32_t sb = s0s[q] + g * G;
          if (sb >= 0 && sb < lens[q])
            *reinterpret_cast<gran_t*>(stage + ads[q] + g * G) = load_vec<G, false>(base + offs[q] + g * G);
        }
      }
    }
    __syncthreads();
    // ---- staging area -> narrow spans of every narrow-side shard ----
    for (uint32_t e0 = 0; e0 < n_items; e0 += 512u) {
      Block blk[2];
      int32_t s0s[2], lens[2];
      uint32_t vks[2], js[2];
      bool anys[2];
#pragma unroll
      for (int q = 0; q < 2; ++q) {
        const uint32_t e = e0 + (uint32_t)q * 256u + tid;
        REDIST_SPAN_ITEM(e, vk, j, s0, len, sb, lim, any)
        (void)lim;
        s0s[q] = s0; lens[q] = len; vks[q] = vk; js[q] = j; anys[q] = any;
        if (!any) continue;
        REDIST_SPAN_FIRST(s0, sb, g0, ad, col)
#pragma unroll
        for (int g = 0; g < GP; ++g) {
          if (g < g0) continue;
          if (s0 + g * G < len) blk[q].g[g] = *reinterpret_cast<const gran_t*>(stage + ad);
          REDIST_SPAN_NEXT(ad, col)
        }
      }
#pragma unroll
      for (int q = 0; q < 2; ++q) {
        if (!anys[q]) continue;
        const bool full = s0s[q] >= 0 && s0s[q] + 16 <= lens[q];
        for (uint32_t jn = jn_first; jn < jn_end; ++jn) {
          char* p = s_nptr[vks[q] * narrow_count + jn] + ((int64_t)js[q] << 4);
          if (full) {
            store_vec<16, true>(p, blk[q].v);
          } else {
#pragma unroll
            for (int g = 0; g < GP; ++g) {
              const int32_t sb = s0s[q] + g * G;
              if (sb >= 0 && sb < lens[q]) store_vec<G, false>(p + g * G, blk[q].g[g]);
            }
          }
        }
      }
    }
  }
#undef REDIST_SPAN_FIRST
#undef REDIST_SPAN_NEXT
#undef REDIST_SPAN_ITEM
#undef REDIST_SPAN_WITEM
}

#define REDIST_ROW_KERNEL(name)                                                              \
  template <int VN, int DIR, class PT>                                                       \
  __global__ void __launch_bounds__(256) name(RowArgs a, PT src, PT dst) {                   \
    row_tile<VN, DIR, PT>(a, src, dst);                                                      \
  }                                                                                          \
  template <int VN, int DIR, class PT>                                                       \
  __global__ void __launch_bounds__(256) name##_t(RowArgs a, PT src, PT dst) {               \
    row_tile<VN, DIR, PT, 1024>(a, src, dst);                                                \
  }                                                                                          \
  template <int VN, int DIR, class PT>                                                       \
  __global__ void __launch_bounds__(256) name##_d(RowArgs a, PT src, PT dst) {               \
    row_tile<VN, DIR, PT, 256, true>(a, src, dst);                                           \
  }                                                                                          \
  template <int VW, int V, int DIR, class PT>                                                \
  __global__ void __launch_bounds__(256) name##_g(RowArgs a, PT src, PT dst) {               \
    row_tile_general<VW, V, DIR, PT>(a, src, dst);                                           \
  }                                                                                          \
  template <int G, int DIR, class PT>                                                        \
  __global__ void __launch_bounds__(256) name##_s(RowArgs a, PT src, PT dst) {               \
    row_tile_span<G, DIR, PT>(a, src, dst);                                                  \
  }                                                                                          \
  template <int VW, int V, int DIR, class PT>                                                \
  __global__ void __launch_bounds__(256) name##_gd(RowArgs a, PT src, PT dst) {              \
    row_tile_general<VW, V, DIR, PT, true>(a, src, dst);                                     \
  }                                                                                          \
  template <int G, int DIR, class PT>                                                        \
  __global__ void __launch_bounds__(256) name##_sd(RowArgs a, PT src, PT dst) {              \
    row_tile_span<G, DIR, PT, true>(a, src, dst);                                            \
  }

REDIST_ROW_KERNEL(redist_dynslice_lds_kernel)
REDIST_ROW_KERNEL(redist_allgather_lds_kernel)
REDIST_ROW_KERNEL(redist_alltoall_lds_kernel)
REDIST_ROW_KERNEL(redist_allpermute_lds_kernel)
REDIST_ROW_KERNEL(redist_fused_gather_lds_kernel)

// ---- cell-complete ops: LDS-staged moves for steps that change the tiling of several inner dims ----
struct CellArgs {
  const DevCellBox* __restrict__ boxes;
  const int32_t* __restrict__ dev_list;
  int64_t sstride[kMaxOuter];
  int64_t dstride[kMaxOuter];
  uint32_t n_boxes, n_tiles, tile_base, tiles_per_box, tpb_magic, tpb_shift;
  int32_t n_outer, n_cell, ps, pd, rep, base_first;
  uint32_t rows_per_tile, src_row_bytes, dst_row_bytes, part_pitch;
  uint32_t spv, spv_magic, spv_shift, srow_vecs;     // source vectors per full stretch (reciprocal) and per row
  uint32_t dpv, dpv_magic, dpv_shift, drow_vecs;     // the same for a destination part
  uint32_t drow_gran, drg_magic, drg_shift;
  uint32_t dext[kMaxCellDims], dext_magic[kMaxCellDims], dext_shift[kMaxCellDims];
  uint32_t piece[kMaxCellDims], piece_magic[kMaxCellDims], piece_shift[kMaxCellDims];
  uint32_t lds_step[kMaxCellDims], part_step[kMaxCellDims];
};

// Where granule x of the last cell dim lies in the staging area, relative to the row's other terms.
__device__ __forceinline__ uint32_t cell_last_term(const CellArgs& a, uint32_t x) {
  uint32_t addr = 0;
  if (a.piece[0]) {
    const uint32_t p = a.piece[0] == 1u ? x : (__umulhi(x, a.piece_magic[0]) >> a.piece_shift[0]);
    x -= p * a.piece[0];
    addr = p * a.part_step[0];
  }
  return addr + x * a.lds_step[0];
}

// Granule gi of a destination part's stretch (rows of drow_gran granules) -> staging address without the last
// dim's term, and the granule's index along the last dim.
__device__ __forceinline__ uint32_t cell_row_terms(const CellArgs& a, uint32_t base, uint32_t gi, uint32_t* x0_out) {
  const uint32_t row = a.drow_gran == 1u ? gi : (__umulhi(gi, a.drg_magic) >> a.drg_shift);
  uint32_t jj = gi - row * a.drow_gran;
  uint32_t addr = base + row * a.src_row_bytes;
  if (a.n_cell == 1) {                      // the last dim is the whole row
    *x0_out = jj;
  } else {
    const uint32_t q = a.dext[0] == 1u ? jj : (__umulhi(jj, a.dext_magic[0]) >> a.dext_shift[0]);
    *x0_out = jj - q * a.dext[0];
    jj = q;
  }
#pragma unroll
  for (int i = 1; i < kMaxCellDims; ++i) {
    if (i < a.n_cell) {
      uint32_t x = jj;
      if (i + 1 < a.n_cell) {
        const uint32_t q = a.dext[i] == 1u ? jj : (__umulhi(jj, a.dext_magic[i]) >> a.dext_shift[i]);
        x = jj - q * a.dext[i];
        jj = q;
      }
      if (a.piece[i]) {
        const uint32_t p = a.piece[i] == 1u ? x : (__umulhi(x, a.piece_magic[i]) >> a.piece_shift[i]);
        x -= p * a.piece[i];
        addr += p * a.part_step[i];
      }
      addr += x * a.lds_step[i];
    }
  }
  return addr;
}

// One tile: rows_per_tile consecutive rows of a box.  Every source part contributes one contiguous stretch, staged
// part after part (part_pitch bytes apart); every destination part receives one contiguous stretch, whose vectors
// are put together from granules of G bytes found in the staging area by the digits of their position in the cell.
template <int VS, int VD, int G, class PT>
__device__ __forceinline__ void cell_tile(const CellArgs& a, const PT& src, const PT& dst) {
  typedef typename VecOf<VS>::type vecs_t;
  typedef typename VecOf<VD>::type vecd_t;
  typedef typename VecOf<G>::type gran_t;
  static_assert(VS % G == 0 && VD % G == 0, "side vectors are whole granules");
  __shared__ __align__(16) unsigned char stage[kCellTileBytes];
  __shared__ char* s_sptr[kCellMaxParts];
  __shared__ char* s_dptr[kCellMaxParts];
  __shared__ uint32_t s_base[kCellMaxParts];

  const uint32_t tile = blockIdx.x + a.tile_base;
  if (tile >= a.n_tiles) return;
  uint32_t b;
  if (a.tiles_per_box) {
    b = a.tiles_per_box == 1u ? tile : (__umulhi(tile, a.tpb_magic) >> a.tpb_shift);
  } else {
    uint32_t lo = 0, hi = a.n_boxes - 1;
    while (lo < hi) {
      uint32_t mid = (lo + hi + 1) >> 1;
      if (a.boxes[mid].tile_first <= tile) lo = mid; else hi = mid - 1;
    }
    b = lo;
  }
  const DevCellBox& bx = a.boxes[b];
  const uint32_t tid = threadIdx.x;
  const int n_outer = a.n_outer;
  // block-uniform: which rows, and where they start on both sides
  const uint32_t tb = tile - bx.tile_first;
  uint32_t rest = bx.row_tiles == 1u ? tb : (__umulhi(tb, bx.rt_magic) >> bx.rt_shift);
  const uint32_t row0 = (tb - rest * bx.row_tiles) * a.rows_per_tile;
  const uint32_t rows = min(a.rows_per_tile, bx.len[n_outer - 1] - row0);
  int64_t so = bx.src_off + (int64_t)row0 * a.src_row_bytes, dof = bx.dst_off + (int64_t)row0 * a.dst_row_bytes;
  for (int k = n_outer - 2; k > 0; --k) {
    const uint32_t len = bx.len[k];
    const uint32_t q = len == 1u ? rest : (__umulhi(rest, bx.magic[k]) >> shift_of(bx, k));
    const uint32_t idx = rest - q * len;
    so += (int64_t)idx * a.sstride[k];
    dof += (int64_t)idx * a.dstride[k];
    rest = q;
  }
  if (n_outer > 1) {
    so += (int64_t)rest * a.sstride[0];
    dof += (int64_t)rest * a.dstride[0];
  }
  const uint32_t ps = (uint32_t)a.ps, pd = (uint32_t)a.pd, rep = (uint32_t)a.rep;
  if (tid < ps) s_sptr[tid] = static_cast<char*>(src.at(a.dev_list[bx.src_first + (int32_t)tid])) + so;
  if (tid < pd * rep) s_dptr[tid] = static_cast<char*>(dst.at(a.dev_list[bx.dst_first + (int32_t)tid])) + dof;
  if (tid < pd) s_base[tid] = (uint32_t)a.dev_list[a.base_first + (int32_t)tid];
  __syncthreads();

  const bool full = rows == a.rows_per_tile;
  // ---- every source part's stretch -> staging area ----
  {
    const uint32_t spv = full ? a.spv : rows * a.srow_vecs, total = ps * spv;
    for (uint32_t e0 = 0; e0 < total; e0 += 1024u) {
      vecs_t v[4];
      uint32_t addr[4];
      bool ok[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const uint32_t e = e0 + (uint32_t)q * 256u + tid;
        ok[q] = e < total;
        const uint32_t s = !ok[q] || ps == 1u ? 0u : full ? (spv == 1u ? e : (__umulhi(e, a.spv_magic) >> a.spv_shift)) : e / spv;
        const uint32_t i = ok[q] ? e - s * spv : 0u;
        addr[q] = s * a.part_pitch + i * (uint32_t)VS;
        v[q] = load_vec<VS, true>(s_sptr[s] + (int64_t)(i * (uint32_t)VS));
      }
#pragma unroll
      for (int q = 0; q < 4; ++q)
        if (ok[q]) *reinterpret_cast<vecs_t*>(stage + addr[q]) = v[q];
    }
  }
  __syncthreads();
  // ---- staging area -> every destination part's stretch ----
  {
    const uint32_t dpv = full ? a.dpv : rows * a.drow_vecs, total = pd * dpv;
    constexpr uint32_t GPV = (uint32_t)(VD / G);   // granules per destination vector
    for (uint32_t e0 = 0; e0 < total; e0 += 256u) {
      const uint32_t e = e0 + tid;
      if (e < total) {
        const uint32_t q = pd == 1u ? 0u : full ? (dpv == 1u ? e : (__umulhi(e, a.dpv_magic) >> a.dpv_shift)) : e / dpv;
        const uint32_t i = e - q * dpv;
        const uint32_t base = s_base[q];
        union { vecd_t v; gran_t g[GPV]; } u;
        uint32_t x0;
        const uint32_t hi = cell_row_terms(a, base, i * GPV, &x0);
        u.g[0] = *reinterpret_cast<const gran_t*>(stage + hi + cell_last_term(a, x0));
#pragma unroll
        for (uint32_t k = 1; k < GPV; ++k) {
          uint32_t at;
          if (x0 + k < a.dext[0]) {           // still in the same row of the last dim
            at = hi + cell_last_term(a, x0 + k);
          } else {
            uint32_t x1;
            const uint32_t hi1 = cell_row_terms(a, base, i * GPV + k, &x1);
            at = hi1 + cell_last_term(a, x1);
          }
          u.g[k] = *reinterpret_cast<const gran_t*>(stage + at);
        }
        char* const* dp = s_dptr + q * rep;
        const int64_t o = (int64_t)(i * (uint32_t)VD);
        for (uint32_t j = 0; j < rep; ++j) store_vec<VD, true>(dp[j] + o, u.v);
      }
    }
  }
}

#define REDIST_CELL_KERNEL(name)                                                             \
  template <int VS, int VD, int G, class PT>                                                 \
  __global__ void __launch_bounds__(256) name(CellArgs a, PT src, PT dst) {                  \
    cell_tile<VS, VD, G, PT>(a, src, dst);                                                   \
  }
REDIST_CELL_KERNEL(redist_dynslice_cell_kernel)
REDIST_CELL_KERNEL(redist_allgather_cell_kernel)
REDIST_CELL_KERNEL(redist_alltoall_cell_kernel)
REDIST_CELL_KERNEL(redist_allpermute_cell_kernel)
REDIST_CELL_KERNEL(redist_fused_gather_cell_kernel)

typedef VecOf<16>::type vec16_t;
constexpr int kUnroll = 8;

__global__ void __launch_bounds__(256) redist_copy_kernel(vec16_t* __restrict__ dst, const vec16_t* __restrict__ src,
                                                          int64_t n_vec) {
  const int64_t base = (int64_t)blockIdx.x * (256 * kUnroll) + threadIdx.x;
  vec16_t v[kUnroll];
  if (base - threadIdx.x + 256 * kUnroll <= n_vec) {  // whole tile in range (block-uniform)
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) v[u] = __builtin_nontemporal_load(src + base + u * 256);
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) __builtin_nontemporal_store(v[u], dst + base + u * 256);
  } else {
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      const int64_t i = base + (int64_t)u * 256;
      if (i < n_vec) __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
    }
  }
}

// An op with more tiles than one grid may have workgroups (the runtime refuses 2^32 threads and more per grid
// dimension) goes out as several launches, each told the launch index of its first workgroup.
template <int V, int U, bool NT, int DM, class PS, class PD>
static hipError_t launch_pt(int kind, OpArgs a, uint32_t max_grid, const PS& src, const PD& dst, hipStream_t stream) {
  for (uint64_t base = 0; base < a.n_tiles; base += max_grid) {
    a.tile_base = (uint32_t)base;
    if (DM > 0) {   // the copies the destination-major body reads
      uint32_t* h = reinterpret_cast<uint32_t*>(&a.hot);
      const uint64_t bp = (uint64_t)(uintptr_t)a.boxes, lp = (uint64_t)(uintptr_t)a.dst_list;
      const uint64_t s0 = (uint64_t)a.sstride[0], d0 = (uint64_t)a.dstride[0];
      h[kH_n_tiles] = a.n_tiles; h[kH_tile_base] = a.tile_base; h[kH_chunk_tiles] = a.chunk_tiles; h[kH_src_tiles] = a.src_tiles;
      h[kH_dm_count] = a.dm_count; h[kH_dm_magic] = a.dm_magic; h[kH_dm_shift] = a.dm_shift; h[kH_dm_dests] = a.dm_dests;
      h[kH_tiles_per_box] = a.tiles_per_box; h[kH_tpb_magic] = a.tpb_magic; h[kH_tpb_shift] = a.tpb_shift; h[kH_n_boxes] = a.n_boxes;
      h[kH_tc] = a.tc; h[kH_tr] = a.tr; h[kH_tc_magic] = a.tc_magic; h[kH_tc_shift] = a.tc_shift;
      uint32_t* g = h + 16;
      g[kG_n_outer] = (uint32_t)a.n_outer; g[kG_common_first] = (uint32_t)a.dm_common_first;
      g[kG_sib_count] = a.sib_count; g[kG_sib_magic] = a.sib_magic; g[kG_sib_shift] = a.sib_shift;
      g[kG_sib_group_tiles] = a.sib_group_tiles; g[kG_sib_gt_magic] = a.sib_gt_magic; g[kG_sib_gt_shift] = a.sib_gt_shift;
      g[kG_boxes_lo] = (uint32_t)bp; g[kG_boxes_hi] = (uint32_t)(bp >> 32); g[kG_list_lo] = (uint32_t)lp; g[kG_list_hi] = (uint32_t)(lp >> 32);
      g[kG_ss0_lo] = (uint32_t)s0; g[kG_ss0_hi] = (uint32_t)(s0 >> 32); g[kG_ds0_lo] = (uint32_t)d0; g[kG_ds0_hi] = (uint32_t)(d0 >> 32);
    }
    dim3 grid((uint32_t)std::min<uint64_t>(max_grid, a.n_tiles - base)), block(256);
    switch (kind) {
      case 0: hipLaunchKernelGGL((redist_dynslice_kernel<V, U, NT, DM, PS, PD>), grid, block, 0, stream, a, src, dst); break;
      case 1: hipLaunchKernelGGL((redist_allgather_kernel<V, U, NT, DM, PS, PD>), grid, block, 0, stream, a, src, dst); break;
      case 2: hipLaunchKernelGGL((redist_alltoall_kernel<V, U, NT, DM, PS, PD>), grid, block, 0, stream, a, src, dst); break;
      case 3: hipLaunchKernelGGL((redist_allpermute_kernel<V, U, NT, DM, PS, PD>), grid, block, 0, stream, a, src, dst); break;
      default: hipLaunchKernelGGL((redist_fused_gather_kernel<V, U, NT, DM, PS, PD>), grid, block, 0, stream, a, src, dst); break;
    }
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

template <int V, int U, bool NT, int DM>
static hipError_t launch_v(int kind, const OpArgs& a, uint32_t max_grid, const PtrTable& src, const PtrTable& dst,
                           hipStream_t stream) {
  if (src.ext)
    return launch_pt<V, U, NT, DM, PtrTableExt, PtrTableExt>(kind, a, max_grid, PtrTableExt{src.ext}, PtrTableExt{dst.ext}, stream);
  return launch_pt<V, U, NT, DM, PtrTable, PtrTable>(kind, a, max_grid, src, dst, stream);
}

int launch_copy_op(const CopyOp& op, const void* dev_boxes, const void* dev_dst_list, const PtrTable& src,
                   const PtrTable& dst, void* stream) {
  if (op.n_tiles == 0) return 0;
  OpArgs a;
  a.boxes = static_cast<const DevBox*>(dev_boxes);
  a.dst_list = static_cast<const int32_t*>(dev_dst_list);
  for (int k = 0; k < kMaxOuter; ++k) { a.sstride[k] = op.sstride[k]; a.dstride[k] = op.dstride[k]; }
  a.n_boxes = (uint32_t)op.boxes.size();
  a.n_tiles = op.n_tiles;
  a.tiles_per_box = op.tiles_per_box;
  a.tpb_magic = op.tpb_magic;
  a.tpb_shift = op.tpb_shift;
  a.n_outer = op.n_outer;
  a.tc = (uint32_t)op.tc;
  a.tr = (uint32_t)op.tr;
  a.tc_magic = op.tc_magic;
  a.tc_shift = op.tc_shift;
  hipStream_t s = static_cast<hipStream_t>(stream);
  hipError_t e;
  a.chunk_tiles = op.chunk_tiles;
  a.src_tiles = op.src_tiles;
  a.dm_count = op.dm_groups;    // what the launch index is divided by
  a.dm_dests = op.dm_count;
  a.dm_magic = op.dm_magic;
  a.dm_shift = op.dm_shift;
  a.dm_common_first = -1;
  if (op.dest_major && !op.boxes.empty()) {
    a.dm_common_first = op.boxes.front().dst_first;
    for (const DevBox& b : op.boxes)
      if (b.dst_first != op.boxes.front().dst_first) a.dm_common_first = -1;
  }
  a.tile_base = 0;
  a.sib_count = op.sib_count; a.sib_magic = op.sib_magic; a.sib_shift = op.sib_shift | (op.sib_inner_log2 << 8);
  a.sib_group_tiles = op.sib_count * op.tiles_per_box;
  a.sib_gt_magic = 0; a.sib_gt_shift = 0;
  const uint32_t mg = op.max_grid;
  const int key = op.vec_bytes == 16 ? op.unroll : -op.vec_bytes;
  if (op.sib_count > 1) {
    // what the kernel assumes about sibling boxes, checked once more where the launch is made
    if (key != 1 || op.tiles_per_box == 0 || op.boxes.size() % op.sib_count ||
        (op.dest_major && op.dm_fanout != 1 && op.dm_fanout != 2))
      return (int)hipErrorInvalidValue;
    for (const DevBox& b : op.boxes)
      if (b.n_tiles != op.tiles_per_box) return (int)hipErrorInvalidValue;
    uint8_t sh = 0;
    magic_for(a.sib_group_tiles, &a.sib_gt_magic, &sh);
    a.sib_gt_shift = sh;
    if (op.sib_inner_log2 == 0)
      e = !op.dest_major ? launch_v<16, 1, true, -1>(op.kind, a, mg, src, dst, s)
          : op.dm_fanout == 2 ? launch_v<16, 1, true, 4>(op.kind, a, mg, src, dst, s)
                              : launch_v<16, 1, true, 3>(op.kind, a, mg, src, dst, s);
    else
      e = !op.dest_major ? launch_v<16, 1, true, -2>(op.kind, a, mg, src, dst, s)
          : op.dm_fanout == 2 ? launch_v<16, 1, true, 6>(op.kind, a, mg, src, dst, s)
                              : launch_v<16, 1, true, 5>(op.kind, a, mg, src, dst, s);
    return (int)e;
  }
  if (op.dest_major) {   // one vector per thread for 16-byte vectors (the builder sees to it)
    if (op.dm_fanout == 2) {
      switch (key) {
        case 1: e = launch_v<16, 1, true, 2>(op.kind, a, mg, src, dst, s); break;
        case -8: e = launch_v<8, 4, true, 2>(op.kind, a, mg, src, dst, s); break;
        case -4: e = launch_v<4, 4, true, 2>(op.kind, a, mg, src, dst, s); break;
        case -2: e = launch_v<2, 4, true, 2>(op.kind, a, mg, src, dst, s); break;
        case -1: e = launch_v<1, 4, true, 2>(op.kind, a, mg, src, dst, s); break;
        default: e = hipErrorInvalidValue; break;
      }
      return (int)e;
    }
    if (op.dm_fanout != 1) return (int)hipErrorInvalidValue;
    switch (key) {
      case 1: e = launch_v<16, 1, true, 1>(op.kind, a, mg, src, dst, s); break;
      case -8: e = launch_v<8, 4, true, 1>(op.kind, a, mg, src, dst, s); break;
      case -4: e = launch_v<4, 4, true, 1>(op.kind, a, mg, src, dst, s); break;
      case -2: e = launch_v<2, 4, true, 1>(op.kind, a, mg, src, dst, s); break;
      case -1: e = launch_v<1, 4, true, 1>(op.kind, a, mg, src, dst, s); break;
      default: e = hipErrorInvalidValue; break;
    }
    return (int)e;
  }
  switch (key) {
    case 1: e = launch_v<16, 1, true, 0>(op.kind, a, mg, src, dst, s); break;
    case 2: e = launch_v<16, 2, true, 0>(op.kind, a, mg, src, dst, s); break;
    case 4: e = launch_v<16, 4, true, 0>(op.kind, a, mg, src, dst, s); break;
    case 8: e = launch_v<16, 8, true, 0>(op.kind, a, mg, src, dst, s); break;
    case -8: e = launch_v<8, 4, true, 0>(op.kind, a, mg, src, dst, s); break;
    case -4: e = launch_v<4, 4, true, 0>(op.kind, a, mg, src, dst, s); break;
    case -2: e = launch_v<2, 4, true, 0>(op.kind, a, mg, src, dst, s); break;
    default: e = launch_v<1, 4, true, 0>(op.kind, a, mg, src, dst, s); break;
  }
  return (int)e;
}

// Row-complete ops split over several launches like the generic ones (see launch_pt): `one` enqueues one launch.
template <class F>
static hipError_t launch_row_split(RowArgs a, uint32_t max_grid, F&& one) {
  for (uint64_t base = 0; base < a.n_tiles; base += max_grid) {
    a.tile_base = (uint32_t)base;
    one(a, dim3((uint32_t)std::min<uint64_t>(max_grid, a.n_tiles - base)));
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

// the five entry points of one form of the staged body, chosen by the step kind
#define REDIST_ROW_LAUNCH(suffix, ...)                                                                                   \
  switch (kind) {                                                                                                        \
    case 0: hipLaunchKernelGGL((redist_dynslice_lds_kernel##suffix<__VA_ARGS__>), grid, dim3(256), 0, stream, ra, src, dst); break;    \
    case 1: hipLaunchKernelGGL((redist_allgather_lds_kernel##suffix<__VA_ARGS__>), grid, dim3(256), 0, stream, ra, src, dst); break;   \
    case 2: hipLaunchKernelGGL((redist_alltoall_lds_kernel##suffix<__VA_ARGS__>), grid, dim3(256), 0, stream, ra, src, dst); break;    \
    case 3: hipLaunchKernelGGL((redist_allpermute_lds_kernel##suffix<__VA_ARGS__>), grid, dim3(256), 0, stream, ra, src, dst); break;  \
    default: hipLaunchKernelGGL((redist_fused_gather_lds_kernel##suffix<__VA_ARGS__>), grid, dim3(256), 0, stream, ra, src, dst); break; \
  }

template <int VN, int DIR, class PT>
static hipError_t launch_row_pt(int kind, const RowArgs& a, uint32_t max_grid, const PT& src, const PT& dst,
                                hipStream_t stream, int general_vw) {
  // (destination-major order: the host chooses it only where pointers travel as arguments)
  const bool dm = a.dm_dests > 1;
  if (dm && !std::is_same<PT, PtrTable>::value) return hipErrorInvalidValue;
  if (general_vw < 0) {   // span form
    if constexpr (VN < 16) {
      if constexpr (std::is_same<PT, PtrTable>::value)
        if (dm) return launch_row_split(a, max_grid, [&](const RowArgs& ra, dim3 grid) { REDIST_ROW_LAUNCH(_sd, VN, DIR, PT) });
      return launch_row_split(a, max_grid, [&](const RowArgs& ra, dim3 grid) { REDIST_ROW_LAUNCH(_s, VN, DIR, PT) });
    } else {
      return hipErrorInvalidValue;
    }
  }
  if (general_vw == 16) {
    if constexpr (std::is_same<PT, PtrTable>::value)
      if (dm) return launch_row_split(a, max_grid, [&](const RowArgs& ra, dim3 grid) { REDIST_ROW_LAUNCH(_gd, 16, VN, DIR, PT) });
    return launch_row_split(a, max_grid, [&](const RowArgs& ra, dim3 grid) { REDIST_ROW_LAUNCH(_g, 16, VN, DIR, PT) });
  }
  if (general_vw > 0) {
    if constexpr (std::is_same<PT, PtrTable>::value)
      if (dm) return launch_row_split(a, max_grid, [&](const RowArgs& ra, dim3 grid) { REDIST_ROW_LAUNCH(_gd, VN, VN, DIR, PT) });
    return launch_row_split(a, max_grid, [&](const RowArgs& ra, dim3 grid) { REDIST_ROW_LAUNCH(_g, VN, VN, DIR, PT) });
  }
  if (dm) {   // destination-major order (the host chooses it only where pointers travel as arguments)
    if constexpr (std::is_same<PT, PtrTable>::value)
      return launch_row_split(a, max_grid, [&](const RowArgs& ra, dim3 grid) { REDIST_ROW_LAUNCH(_d, VN, DIR, PT) });
    else
      return hipErrorInvalidValue;
  }
  if (a.r_log2 > 8)   // tiles of more than 256 rows: wide rows of 16 or 32 bytes
    return launch_row_split(a, max_grid, [&](const RowArgs& ra, dim3 grid) { REDIST_ROW_LAUNCH(_t, VN, DIR, PT) });
  return launch_row_split(a, max_grid, [&](const RowArgs& ra, dim3 grid) { REDIST_ROW_LAUNCH(, VN, DIR, PT) });
}
#undef REDIST_ROW_LAUNCH

template <int VN, int DIR>
static hipError_t launch_row_v(int kind, const RowArgs& a, uint32_t max_grid, const PtrTable& src, const PtrTable& dst,
                               hipStream_t stream, int general_vw) {
  if (src.ext)
    return launch_row_pt<VN, DIR, PtrTableExt>(kind, a, max_grid, PtrTableExt{src.ext}, PtrTableExt{dst.ext}, stream, general_vw);
  return launch_row_pt<VN, DIR, PtrTable>(kind, a, max_grid, src, dst, stream, general_vw);
}

int launch_row_op(int kind, const RowOp& op, const void* dev_boxes, const void* dev_pieces, const void* dev_list,
                  const PtrTable& src, const PtrTable& dst, void* stream) {
  if (op.n_tiles == 0) return 0;
  RowArgs a;
  a.boxes = static_cast<const DevRowBox*>(dev_boxes);
  a.pieces = static_cast<const DevPiece*>(dev_pieces);
  a.dev_list = static_cast<const int32_t*>(dev_list);
  for (int k = 0; k < kMaxOuter; ++k) { a.wstride[k] = op.wstride[k]; a.nstride[k] = op.nstride[k]; }
  a.n_boxes = (uint32_t)op.boxes.size();
  a.n_tiles = op.n_tiles;
  a.tiles_per_box = op.tiles_per_box;
  a.tpb_magic = op.tpb_magic;
  a.tpb_shift = op.tpb_shift;
  a.n_outer = op.n_outer;
  a.w_log2 = op.w_log2;
  a.n_log2 = op.n_log2;
  a.r_log2 = op.r_log2;
  a.n_pieces = op.n_pieces;
  a.narrow_count = op.narrow_count;
  a.n_bytes = op.n_bytes; a.pitch = op.pitch;
  a.cpn = op.cpn; a.cpn_magic = op.cpn_magic; a.cpn_shift = op.cpn_shift;
  a.wpr = op.wpr; a.wpr_magic = op.wpr_magic; a.wpr_shift = op.wpr_shift;
  a.w_bytes = op.w_bytes; a.rpt = op.rpt; a.rpt_magic = op.rpt_magic; a.rpt_shift = op.rpt_shift;
  a.nbm = op.nbm; a.nbm_magic = op.nbm_magic; a.nbm_shift = op.nbm_shift;
  a.w_shard_bytes = op.wide_shard_bytes; a.n_shard_bytes = op.narrow_shard_bytes;
  a.mct = op.mct; a.slot = op.slot; a.cbw = op.cbw; a.cbw_magic = op.cbw_magic; a.cbw_shift = op.cbw_shift;
  a.chunk_dims = op.chunk_dims;
  a.dm_count = op.dm_groups; a.dm_magic = op.dm_magic; a.dm_shift = op.dm_shift;
  a.dm_fanout = op.dm_fanout; a.dm_dests = op.dm_count;
  a.chunk_tiles = op.chunk_tiles; a.src_tiles = op.src_tiles;
  a.tile_base = 0;
  hipStream_t s = static_cast<hipStream_t>(stream);
  hipError_t e;
  // general form: wide-side vector (16 or vn); span form: -1, granule = vn; power-of-two form: 0
  const int gvw = op.span ? -1 : op.general ? op.vw : 0;
  switch (op.vn * 2 + op.dir) {
    case 32: e = launch_row_v<16, 0>(kind, a, op.max_grid, src, dst, s, gvw); break;
    case 33: e = launch_row_v<16, 1>(kind, a, op.max_grid, src, dst, s, gvw); break;
    case 16: e = launch_row_v<8, 0>(kind, a, op.max_grid, src, dst, s, gvw); break;
    case 17: e = launch_row_v<8, 1>(kind, a, op.max_grid, src, dst, s, gvw); break;
    case 8: e = launch_row_v<4, 0>(kind, a, op.max_grid, src, dst, s, gvw); break;
    case 9: e = launch_row_v<4, 1>(kind, a, op.max_grid, src, dst, s, gvw); break;
    case 4: e = launch_row_v<2, 0>(kind, a, op.max_grid, src, dst, s, gvw); break;
    case 5: e = launch_row_v<2, 1>(kind, a, op.max_grid, src, dst, s, gvw); break;
    case 2: e = launch_row_v<1, 0>(kind, a, op.max_grid, src, dst, s, gvw); break;
    default: e = launch_row_v<1, 1>(kind, a, op.max_grid, src, dst, s, gvw); break;
  }
  return (int)e;
}

// ---- cell-complete ops ----
template <int VS, int VD, int G>
static hipError_t launch_cell_v(int kind, CellArgs a, uint32_t max_grid, const PtrTable& src, const PtrTable& dst,
                                hipStream_t stream) {
  for (uint64_t base = 0; base < a.n_tiles; base += max_grid) {
    a.tile_base = (uint32_t)base;
    const dim3 grid((uint32_t)std::min<uint64_t>(max_grid, a.n_tiles - base));
    switch (kind) {
      case 0: hipLaunchKernelGGL((redist_dynslice_cell_kernel<VS, VD, G, PtrTable>), grid, dim3(256), 0, stream, a, src, dst); break;
      case 1: hipLaunchKernelGGL((redist_allgather_cell_kernel<VS, VD, G, PtrTable>), grid, dim3(256), 0, stream, a, src, dst); break;
      case 2: hipLaunchKernelGGL((redist_alltoall_cell_kernel<VS, VD, G, PtrTable>), grid, dim3(256), 0, stream, a, src, dst); break;
      case 3: hipLaunchKernelGGL((redist_allpermute_cell_kernel<VS, VD, G, PtrTable>), grid, dim3(256), 0, stream, a, src, dst); break;
      default: hipLaunchKernelGGL((redist_fused_gather_cell_kernel<VS, VD, G, PtrTable>), grid, dim3(256), 0, stream, a, src, dst); break;
    }
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

int launch_cell_op(int kind, const CellOp& op, const void* dev_boxes, const void* dev_list, const PtrTable& src,
                   const PtrTable& dst, void* stream) {
  if (op.n_tiles == 0) return 0;
  // what the kernel assumes, checked once more where the launch is made
  if (src.ext || dst.ext || op.ps < 1 || op.pd < 1 || op.ps > kCellMaxParts || op.pd * op.rep > kCellMaxParts ||
      op.n_cell < 1 || op.n_cell > kMaxCellDims || op.n_outer < 1 || op.n_outer > kMaxOuter ||
      (uint64_t)op.ps * op.part_pitch > (uint64_t)kCellTileBytes)
    return (int)hipErrorInvalidValue;
  CellArgs a;
  a.boxes = static_cast<const DevCellBox*>(dev_boxes);
  a.dev_list = static_cast<const int32_t*>(dev_list);
  for (int k = 0; k < kMaxOuter; ++k) { a.sstride[k] = op.sstride[k]; a.dstride[k] = op.dstride[k]; }
  a.n_boxes = (uint32_t)op.boxes.size();
  a.n_tiles = op.n_tiles;
  a.tile_base = 0;
  a.tiles_per_box = op.tiles_per_box; a.tpb_magic = op.tpb_magic; a.tpb_shift = op.tpb_shift;
  a.n_outer = op.n_outer; a.n_cell = op.n_cell; a.ps = op.ps; a.pd = op.pd; a.rep = op.rep; a.base_first = op.base_first;
  a.rows_per_tile = op.rows_per_tile; a.src_row_bytes = op.src_row_bytes; a.dst_row_bytes = op.dst_row_bytes;
  a.part_pitch = op.part_pitch;
  a.spv = op.spv; a.spv_magic = op.spv_magic; a.spv_shift = op.spv_shift; a.srow_vecs = op.src_row_bytes / (uint32_t)op.vs;
  a.dpv = op.dpv; a.dpv_magic = op.dpv_magic; a.dpv_shift = op.dpv_shift; a.drow_vecs = op.dst_row_bytes / (uint32_t)op.vd;
  a.drow_gran = op.drow_gran; a.drg_magic = op.drg_magic; a.drg_shift = op.drg_shift;
  for (int i = 0; i < kMaxCellDims; ++i) {
    a.dext[i] = op.dext[i]; a.dext_magic[i] = op.dext_magic[i]; a.dext_shift[i] = op.dext_shift[i];
    a.piece[i] = op.piece[i]; a.piece_magic[i] = op.piece_magic[i]; a.piece_shift[i] = op.piece_shift[i];
    a.lds_step[i] = op.lds_step[i]; a.part_step[i] = op.part_step[i];
  }
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int key = op.gran * 10000 + op.vs * 100 + op.vd;
  switch (key) {
    case 161616: return (int)launch_cell_v<16, 16, 16>(kind, a, op.max_grid, src, dst, s);
    case 81616: return (int)launch_cell_v<16, 16, 8>(kind, a, op.max_grid, src, dst, s);
    case 81608: return (int)launch_cell_v<16, 8, 8>(kind, a, op.max_grid, src, dst, s);
    case 80816: return (int)launch_cell_v<8, 16, 8>(kind, a, op.max_grid, src, dst, s);
    case 80808: return (int)launch_cell_v<8, 8, 8>(kind, a, op.max_grid, src, dst, s);
    case 41616: return (int)launch_cell_v<16, 16, 4>(kind, a, op.max_grid, src, dst, s);
    case 41604: return (int)launch_cell_v<16, 4, 4>(kind, a, op.max_grid, src, dst, s);
    case 40416: return (int)launch_cell_v<4, 16, 4>(kind, a, op.max_grid, src, dst, s);
    case 40404: return (int)launch_cell_v<4, 4, 4>(kind, a, op.max_grid, src, dst, s);
    default: return (int)hipErrorInvalidValue;
  }
}

// ---- pointer tables of meshes beyond kMaxExecDevices ----
// Such meshes read their shard pointers from device memory.  The tables are written by kernels that carry the
// pointers as arguments, kMaxExecDevices at a time: the refresh is ordered on the caller's stream like every other
// launch, reads no host memory after the call has returned, and can be recorded by a stream capture.
__global__ void __launch_bounds__(kMaxExecDevices) redist_ptr_table_kernel(PtrTable chunk, void** out, int n) {
  const int i = (int)threadIdx.x;
  if (i < n) out[i] = chunk.p[i];
}
// out[d] = base + d * stride: the shards of a workspace region
__global__ void __launch_bounds__(256) redist_ptr_stride_kernel(void** out, char* base, long long stride, int n) {
  const int i = (int)(blockIdx.x * 256u + threadIdx.x);
  if (i < n) out[i] = base + (long long)i * stride;
}

int launch_ptr_table(const void* const* host_ptrs, int n, void** dev_out, void* stream) {
  for (int at = 0; at < n; at += kMaxExecDevices) {
    const int m = n - at < kMaxExecDevices ? n - at : kMaxExecDevices;
    PtrTable chunk{};
    for (int i = 0; i < m; ++i) chunk.p[i] = const_cast<void*>(host_ptrs[at + i]);
    hipLaunchKernelGGL(redist_ptr_table_kernel, dim3(1), dim3(kMaxExecDevices), 0, static_cast<hipStream_t>(stream), chunk,
                       dev_out + at, m);
    const int e = (int)hipGetLastError();
    if (e != 0) return e;
  }
  return 0;
}

int launch_ptr_table_strided(void* base, int64_t stride, int n, void** dev_out, void* stream) {
  if (n <= 0) return 0;
  hipLaunchKernelGGL(redist_ptr_stride_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0,
                     static_cast<hipStream_t>(stream), dev_out, static_cast<char*>(base), (long long)stride, n);
  return (int)hipGetLastError();
}

// ---- fixed scratch area of the entry point that allocates nothing ----
// Part of the library's device image: every GPU the library runs on holds its own copy, at its own address, until
// the process ends.  In host code the array's name is only a handle for hipGetSymbolAddress; kernels and copies get
// the device address that call returns.
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

int static_scratch_base(void** out) {
  constexpr int kMaxGpus = 64;
  static std::mutex mu;
  static void* base[kMaxGpus] = {};
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return (int)e;
  if (dev < 0 || dev >= kMaxGpus) return (int)hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(mu);
  if (!base[dev]) {   // once per device, with that device current
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return (int)e;
    if (!p) return (int)hipErrorInvalidSymbol;
    base[dev] = p;
  }
  *out = base[dev];
  return 0;
}

// Host memory -> device memory with the bytes as kernel arguments, kUploadVecs 16-byte vectors per launch.
constexpr int kUploadVecs = 224;   // 3.5 KiB of the 4 KiB a kernel's arguments may take
struct UploadChunk { vec16_t q[kUploadVecs]; };
__global__ void __launch_bounds__(256) redist_upload_kernel(UploadChunk c, vec16_t* out, int n) {
  const int i = (int)threadIdx.x;
  if (i < n) out[i] = c.q[i];
}

int launch_upload(const void* host_src, size_t bytes, void* dev_dst, void* stream) {
  const char* from = static_cast<const char*>(host_src);
  vec16_t* to = static_cast<vec16_t*>(dev_dst);
  for (size_t at = 0; at < bytes; at += sizeof(UploadChunk)) {
    const size_t here = std::min(sizeof(UploadChunk), bytes - at);
    UploadChunk c;
    std::memset(&c, 0, sizeof(c));
    std::memcpy(&c, from + at, here);
    hipLaunchKernelGGL(redist_upload_kernel, dim3(1), dim3(256), 0, static_cast<hipStream_t>(stream), c,
                       to + at / sizeof(vec16_t), (int)((here + 15) / 16));
    const int e = (int)hipGetLastError();
    if (e != 0) return e;
  }
  return 0;
}

int launch_copy_baseline(void* dst, const void* src, int64_t bytes, void* stream) {
  const int64_t n_vec = bytes / 16;
  if (n_vec == 0) return 0;
  const int64_t per_block = 256 * kUnroll;
  dim3 grid((unsigned)((n_vec + per_block - 1) / per_block)), block(256);
  hipLaunchKernelGGL(redist_copy_kernel, grid, block, 0, static_cast<hipStream_t>(stream), static_cast<vec16_t*>(dst),
                     static_cast<const vec16_t*>(src), n_vec);
  return (int)hipGetLastError();
}

const char* row_kernel_name_of(int kind) {
  switch (kind) {
    case 0: return "redist_dynslice_lds_kernel";
    case 1: return "redist_allgather_lds_kernel";
    case 2: return "redist_alltoall_lds_kernel";
    case 3: return "redist_allpermute_lds_kernel";
    default: return "redist_fused_gather_lds_kernel";
  }
}

const char* cell_kernel_name_of(int kind) {
  switch (kind) {
    case 0: return "redist_dynslice_cell_kernel";
    case 1: return "redist_allgather_cell_kernel";
    case 2: return "redist_alltoall_cell_kernel";
    case 3: return "redist_allpermute_cell_kernel";
    default: return "redist_fused_gather_cell_kernel";
  }
}

const char* kernel_name_of(int kind) {
  switch (kind) {
    case 0: return "redist_dynslice_kernel";
    case 1: return "redist_allgather_kernel";
    case 2: return "redist_alltoall_kernel";
    case 3: return "redist_allpermute_kernel";
    default: return "redist_fused_gather_kernel";
  }
}

}  // namespace redist
