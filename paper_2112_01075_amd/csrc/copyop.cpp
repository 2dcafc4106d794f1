#include "copyop.hpp"

#include <algorithm>
#include <cstdlib>
#include <map>
#include <numeric>

namespace redist {

struct Seg {  // one piece of a destination tile's extent in a dim, lying in one source tile
  int64_t dst_start, len, src_start, src_tile;
};

namespace {

int pow2_floor_gcd(int64_t a, int v) {  // largest power of two <= v dividing a
  while (v > 1 && (a % v)) v >>= 1;
  return v;
}

}  // namespace

void magic_for(uint32_t d, uint32_t* m, uint8_t* s) {
  if (d <= 1) { *m = 0; *s = 0; return; }
  int l = 0;
  while ((1ull << l) < d) ++l;  // ceil(log2 d), 1..32
  unsigned __int128 num = (unsigned __int128)1 << (31 + l);
  uint64_t mm = (uint64_t)((num + d - 1) / d);
  *m = (uint32_t)mm;
  *s = (uint8_t)(l - 1);
}

namespace {
bool build_copy_op_impl(int kind, int ndev, int rank, int elem_size, const std::vector<int64_t>& cs,
                        const std::vector<int64_t>& os, const std::vector<int64_t>& cd, const std::vector<int64_t>& od,
                        const BuildOptions& opt, bool allow_siblings, CopyOp* out);
}  // namespace

bool build_copy_op(int kind, int ndev, int rank, int elem_size, const std::vector<int64_t>& cs,
                   const std::vector<int64_t>& os, const std::vector<int64_t>& cd, const std::vector<int64_t>& od,
                   const BuildOptions& opt, CopyOp* out) {
  if (!build_copy_op_impl(kind, ndev, rank, elem_size, cs, os, cd, od, opt, true, out)) return false;
  // boxes put in source order for an alternation that the tile shapes then did not allow: back to the usual order
  if (out->sib_resorted && out->sib_count <= 1)
    return build_copy_op_impl(kind, ndev, rank, elem_size, cs, os, cd, od, opt, false, out);
  return true;
}

namespace {
bool build_copy_op_impl(int kind, int ndev, int rank, int elem_size, const std::vector<int64_t>& cs,
                        const std::vector<int64_t>& os, const std::vector<int64_t>& cd, const std::vector<int64_t>& od,
                        const BuildOptions& opt, bool allow_siblings, CopyOp* out) {
  CopyOp op;
  op.kind = kind;
  const int r = rank;

  // ---- collapse dims: dim t+1 merges into dim t when it is untouched (same extent in both
  //      tiles, hence a single full segment).  Group g covers original dims [g_lo[g], g_hi[g]].
  std::vector<int> g_lo, g_hi;
  for (int t = 0; t < r; ++t) {
    bool full = cs[t] == cd[t];
    if (t > 0 && full) g_hi.back() = t;
    else { g_lo.push_back(t); g_hi.push_back(t); }
  }
  int ng = (int)g_lo.size();
  std::vector<int64_t> tail(ng, 1), gcs(ng), gcd_(ng);
  for (int g = 0; g < ng; ++g) {
    for (int t = g_lo[g] + 1; t <= g_hi[g]; ++t) tail[g] *= cs[t];
    gcs[g] = cs[g_lo[g]] * tail[g];
    gcd_[g] = cd[g_lo[g]] * tail[g];
  }
  std::vector<int64_t> gss(ng), gds(ng);  // element strides
  {
    int64_t a = 1, b = 1;
    for (int g = ng - 1; g >= 0; --g) { gss[g] = a; gds[g] = b; a *= gcs[g]; b *= gcd_[g]; }
  }

  // ---- destination groups: devices that end with the same tile receive identical bytes ----
  std::map<std::vector<int64_t>, std::vector<int>> dst_groups, holders;
  std::vector<std::vector<int64_t>> order;
  for (int d = 0; d < ndev; ++d) {
    std::vector<int64_t> key(od.begin() + (size_t)d * r, od.begin() + (size_t)(d + 1) * r);
    auto& v = dst_groups[key];
    if (v.empty()) order.push_back(key);
    v.push_back(d);
    holders[std::vector<int64_t>(os.begin() + (size_t)d * r, os.begin() + (size_t)(d + 1) * r)].push_back(d);
  }

  struct HostBox {
    int64_t soff, doff; int src_dev, src_lowest, dst_first, dst_count; std::vector<int64_t> len;
    int grp_dev = 0, sib = 0;   // sibling boxes (see CopyOp::sib_count): source of the group's first box and its
    int64_t grp_soff = 0;       // offset there, and which sibling of the group this box is
  };
  std::vector<HostBox> hb;
  for (const auto& key : order) {
    const std::vector<int>& members = dst_groups[key];
    int dst_first = (int)op.dst_list.size();
    op.dst_list.insert(op.dst_list.end(), members.begin(), members.end());
    // segments per collapsed dim (cut by the source tile boundaries of the group's leading dim)
    std::vector<std::vector<Seg>> segs(ng);
    for (int g = 0; g < ng; ++g) {
      int t = g_lo[g];
      int64_t o = key[t], end = o + cd[t];
      for (int64_t k = o / cs[t]; k * cs[t] < end; ++k) {
        int64_t lo = std::max(o, k * cs[t]), hi = std::min(end, (k + 1) * cs[t]);
        segs[g].push_back(Seg{(lo - o) * tail[g], (hi - lo) * tail[g], (lo - k * cs[t]) * tail[g], k});
      }
    }
    std::vector<size_t> idx(ng, 0);
    while (true) {
      HostBox b;
      b.soff = b.doff = 0;
      b.dst_first = dst_first;
      b.dst_count = (int)members.size();
      std::vector<int64_t> src_key(r);
      for (int g = 0; g < ng; ++g) {
        const Seg& s = segs[g][idx[g]];
        b.soff += s.src_start * gss[g];
        b.doff += s.dst_start * gds[g];
        b.len.push_back(s.len);
        src_key[g_lo[g]] = s.src_tile * cs[g_lo[g]];
        for (int t = g_lo[g] + 1; t <= g_hi[g]; ++t) src_key[t] = key[t];
      }
      auto it = holders.find(src_key);
      if (it == holders.end()) return false;  // source table does not cover the destination tile
      int src = it->second.front();
      for (int h : it->second)  // prefer a holder that is itself a destination (a local slice)
        if (std::find(members.begin(), members.end(), h) != members.end()) { src = h; break; }
      b.src_dev = src;
      b.src_lowest = it->second.front();
      hb.push_back(std::move(b));
      int g = ng - 1;
      while (g >= 0 && ++idx[g] == segs[g].size()) idx[g--] = 0;
      if (g < 0) break;
    }
  }

  // ---- destination-major order (see CopyOp): eligibility, then boxes cut into pieces that are contiguous in
  //      their source shard, in source order ----
  // Ops of 32 MiB and more whose boxes all go to the same number m > 1 of shards.  A chunk of the op (16 MiB of
  // source) is re-read from the L2 once per destination, which it survives only as a dense stretch of memory:
  // pieces that lie a power of two apart share cache sets (measured: 32 pieces of 512 KiB, 4 MiB apart, 3.2 TB/s;
  // the same bytes as whole 4 MiB shards 6.8; stored to all destinations in turn 3.4-4.4).  So (1) every box reads
  // the lowest-numbered holder of its tile -- on one GPU any replica is as near as any other, and a replica that
  // serves every destination is read front to back --, (2) boxes are cut along their outer dims into pieces
  // contiguous in the source (of 16 KiB at least, else the order is not used: measured on the 70 replicating ops
  // among 1000 paper-shaped problems whose pieces are shorter than the 64 KiB asked for before, +4.4 % in the
  // geometric mean and up to +30 % with 16 KiB, nothing beyond -1.2 %; with 4 KiB +5.9 % but one op -28 %, with
  // 1 KiB one op at a third of its rate), and (3) the pieces are sorted by
  // source address.  The destination tiles partition the array, so the pieces read from a shard tile it exactly:
  // the op reads whole shards front to back.
  {
    const int64_t dm_min_bytes = std::max<int64_t>(0, opt.dest_major_min_bytes);
    const bool forced = dm_min_bytes == 0;   // the tests' way to reach this order on small problems
    const int64_t min_piece_bytes = forced ? 0 : (16ll << 10);
    const int m = hb.empty() ? 0 : hb.front().dst_count;
    bool eligible = m > 1 && opt.dest_major;
    int64_t op_elems = 0;
    for (const auto& b : hb) {
      eligible = eligible && b.dst_count == m;
      int64_t n = 1;
      for (int64_t l : b.len) n *= l;
      op_elems += n;
    }
    eligible = eligible && op_elems * elem_size >= dm_min_bytes;
    // Sibling boxes (see CopyOp::sib_count): consecutive boxes of one destination group with the same extents
    // whose runs follow each other in the destination, shorter than a tile is wide, 2 to 8 of them, the same number
    // everywhere.  Each box learns its group (the first sibling's source) and its place in it.
    int sib_p = 1;
    if (eligible && allow_siblings && opt.siblings) {
      const int64_t run1 = hb.front().len[(size_t)ng - 1], run1_bytes = run1 * elem_size;
      bool ok = run1_bytes >= 512 && run1_bytes < opt.sib_max_run;
      int p_all = 0;
      for (size_t i = 0; ok && i < hb.size();) {
        size_t j = i + 1;
        while (j < hb.size() && hb[j].dst_first == hb[i].dst_first && hb[j].len == hb[i].len &&
               hb[j].doff == hb[j - 1].doff + run1)
          ++j;
        const int p = (int)(j - i);
        if (p_all == 0) p_all = p;
        ok = ok && p == p_all && p >= 2 && p <= 8 && hb[i].len[(size_t)ng - 1] == run1;
        for (size_t q = i; q < j; ++q) {
          hb[q].grp_dev = hb[i].src_lowest;
          hb[q].grp_soff = hb[i].soff;
          hb[q].sib = (int)(q - i);
        }
        i = j;
      }
      if (ok && p_all >= 2) sib_p = p_all;
    }
    std::vector<HostBox> pieces;
    if (eligible) {
      for (const auto& b : hb) {
        // the contiguous suffix of the box's dims in the source shard
        int k0 = ng - 1;
        int64_t cnt = b.len[(size_t)ng - 1];
        for (int g = ng - 2; g >= 0; --g) {
          if (b.len[(size_t)g] > 1 && gss[(size_t)g] != cnt) break;
          cnt *= b.len[(size_t)g];
          k0 = g;
        }
        int64_t n_pieces = 1;
        for (int g = 0; g < k0; ++g) n_pieces *= b.len[(size_t)g];
        if (cnt * elem_size < min_piece_bytes || (int64_t)pieces.size() + n_pieces > 65536) { eligible = false; break; }
        std::vector<int64_t> idx((size_t)k0, 0);
        for (int64_t q = 0; q < n_pieces; ++q) {
          HostBox pc = b;
          pc.src_dev = b.src_lowest;
          for (int g = 0; g < k0; ++g) {
            pc.soff += idx[(size_t)g] * gss[(size_t)g];
            pc.grp_soff += idx[(size_t)g] * gss[(size_t)g];
            pc.doff += idx[(size_t)g] * gds[(size_t)g];
            pc.len[(size_t)g] = 1;
          }
          pieces.push_back(std::move(pc));
          for (int g = k0 - 1; g >= 0 && ++idx[(size_t)g] == b.len[(size_t)g]; --g) idx[(size_t)g] = 0;
        }
      }
    }
    if (eligible) {
      // With one group of destinations per workgroup no chunk is read twice, so nothing has to stay in the L2: the
      // pieces then go in destination order, which makes the window of addresses being written dense (sources that
      // alternate inside the destination's rows are taken together).  Measured on the 136 such ops among 1000
      // paper-shaped problems: +1.3 % in the geometric mean, 2 KiB runs of four sources per destination row
      // 4.2 -> 6.25 TB/s, nothing beyond -5 %.  (With several groups the source order wins: what is re-read must
      // be a dense stretch; and cutting pieces finer for a denser window measured -3 % in the mean, -40 % at worst.)
      const int fan = (opt.dm_fanout == 1 || opt.dm_fanout == 2) ? opt.dm_fanout : (m <= 8 ? 2 : 1);
      if (m <= fan)
        std::stable_sort(pieces.begin(), pieces.end(), [](const HostBox& x, const HostBox& y) {
          return x.dst_first != y.dst_first ? x.dst_first < y.dst_first : x.doff < y.doff;
        });
      else if (sib_p > 1 && (op.sib_resorted = true))   // by the group's source, the siblings of a group side by side
        std::stable_sort(pieces.begin(), pieces.end(), [](const HostBox& x, const HostBox& y) {
          if (x.grp_dev != y.grp_dev) return x.grp_dev < y.grp_dev;
          if (x.grp_soff != y.grp_soff) return x.grp_soff < y.grp_soff;
          return x.sib < y.sib;
        });
      else
        std::stable_sort(pieces.begin(), pieces.end(), [](const HostBox& x, const HostBox& y) {
          return x.src_dev != y.src_dev ? x.src_dev < y.src_dev : x.soff < y.soff;
        });
      if (sib_p > 1)   // every group whole and in order?  (else no alternation)
        for (size_t q = 0; q < pieces.size(); ++q)
          if (pieces[q].sib != (int)(q % (size_t)sib_p) || pieces[q].grp_soff != pieces[q - (size_t)pieces[q].sib].grp_soff ||
              pieces[q].grp_dev != pieces[q - (size_t)pieces[q].sib].grp_dev) { sib_p = 1; break; }
      hb = std::move(pieces);
      op.dest_major = true;
    }
    if (op.dest_major && sib_p > 1) op.sib_count = (uint32_t)sib_p;
  }

  // ---- ordinary order: sibling boxes of either side (see CopyOp::sib_count) ----
  // Boxes of one shape whose runs (512 bytes to under 4 KiB) follow each other in the destination's rows -- they stand
  // side by side already -- or else in the source's rows, for which the boxes are first put in source order.  Chains
  // of more than 8 such boxes alternate in groups of 8, 4 or 2.
  if (!op.dest_major && allow_siblings && opt.siblings && hb.size() >= 2) {
    const int64_t run1 = hb.front().len[(size_t)ng - 1], run1_bytes = run1 * elem_size;
    auto chains_of = [&](const std::vector<HostBox>& v, bool by_dst) -> int {
      size_t len_all = 0;
      for (size_t i = 0; i < v.size();) {
        size_t j = i + 1;
        while (j < v.size() && v[j].len == v[i].len &&
               (by_dst ? v[j].dst_first == v[i].dst_first && v[j].doff == v[j - 1].doff + run1
                       : v[j].src_dev == v[i].src_dev && v[j].soff == v[j - 1].soff + run1))
          ++j;
        if (len_all == 0) len_all = j - i;
        if (j - i != len_all || len_all < 2 || v[i].len[(size_t)ng - 1] != run1) return 1;
        i = j;
      }
      if (len_all <= 8) return (int)len_all;
      return len_all % 8 == 0 ? 8 : len_all % 4 == 0 ? 4 : len_all % 2 == 0 ? 2 : 1;
    };
    if (run1_bytes >= 512 && run1_bytes < opt.sib_max_run) {
      int p = chains_of(hb, true);
      if (p < 2 && run1_bytes < 4096) {   // (pieces of the source's rows: only short ones gain)
        std::vector<HostBox> by_src = hb;
        std::stable_sort(by_src.begin(), by_src.end(), [](const HostBox& x, const HostBox& y) {
          return x.src_dev != y.src_dev ? x.src_dev < y.src_dev : x.soff < y.soff;
        });
        p = chains_of(by_src, false);
        if (p >= 2) { hb = std::move(by_src); op.sib_resorted = true; }
      }
      if (p >= 2) op.sib_count = (uint32_t)p;
    }
  }

  // ---- drop outer dims of extent 1 everywhere; last collapsed dim is the run ----
  std::vector<int> keep;
  for (int g = 0; g < ng - 1; ++g) {
    bool all_one = true;
    for (const auto& b : hb) all_one = all_one && b.len[g] == 1;
    if (!all_one) keep.push_back(g);
  }
  op.n_outer = (int)keep.size();
  if (op.n_outer > kMaxOuter) return false;
  for (int k = 0; k < kMaxOuter; ++k) { op.sstride[k] = 0; op.dstride[k] = 0; }
  for (int k = 0; k < op.n_outer; ++k) {
    op.sstride[k] = gss[keep[k]] * elem_size;
    op.dstride[k] = gds[keep[k]] * elem_size;
  }

  // ---- vector width: every run, offset and stride must be a multiple of it ----
  int v = 16;
  for (int k = 0; k < op.n_outer; ++k) { v = pow2_floor_gcd(op.sstride[k], v); v = pow2_floor_gcd(op.dstride[k], v); }
  int64_t max_run_bytes = 0;
  for (const auto& b : hb) {
    int64_t run_bytes = b.len[ng - 1] * elem_size;
    v = pow2_floor_gcd(run_bytes, v);
    v = pow2_floor_gcd(b.soff * elem_size, v);
    v = pow2_floor_gcd(b.doff * elem_size, v);
    max_run_bytes = std::max(max_run_bytes, run_bytes);
  }
  if (op.sib_count > 1 && v != 16) op.sib_count = 1;   // (the alternating kernel is instantiated for 16-byte vectors)
  op.vec_bytes = v;

  // ---- tiling: 256 threads x unroll vectors; as wide as the longest run allows ----
  int64_t total_vecs = 0;
  for (const auto& b : hb) {
    int64_t n = b.len[ng - 1] * elem_size / v;
    for (int k = 0; k < op.n_outer; ++k) n *= b.len[keep[k]];
    total_vecs += n;
  }
  // Vectors per thread, from measurements on MI355X: one vector (4 KiB tiles) keeps the window of
  // addresses in flight narrow and lets the prologues of later workgroups overlap with transfers,
  // which wins whenever runs are short or medium (2 KiB and 32 KiB runs: +5 %); boxes made of very
  // long runs (whole tiles, MiB-sized pieces) do better with 4.  The caller's options may fix the number.
  op.unroll = max_run_bytes >= (256 << 10) ? 4 : 1;
  const bool unroll_fixed = opt.unroll == 1 || opt.unroll == 2 || opt.unroll == 4 || opt.unroll == 8;
  if (unroll_fixed) op.unroll = opt.unroll;
  op.max_grid = std::max(1u, std::min(opt.max_grid, 16777215u));
  if (op.dest_major || op.sib_count > 1) op.unroll = 1;   // measured: 6.8 TB/s with one vector per thread, 5.9 with two
  int64_t max_run_vecs = std::max<int64_t>(1, max_run_bytes / v);
  // tile width: the longest run cut into equal column blocks (any integer up to the tile size), as
  // many rows as then fit; lanes map to (row, column) by reciprocal division
  const int64_t align_vecs = std::max(1, 128 / v);
  auto shape_of = [&](int u, int extra_blocks, int64_t* tc_out, int64_t* tr_out) {
    const int64_t t = 256 * u, cb_min = (max_run_vecs + t - 1) / t;
    double best = -1.0;
    for (int64_t cb = cb_min; cb <= cb_min + extra_blocks; ++cb) {
      int64_t c = (max_run_vecs + cb - 1) / cb;
      // Column blocks of a run end on 128-byte boundaries of the run.  A boundary inside a 64-byte burst makes two
      // workgroups write part of it each; measured on the 135 of 1000 paper-shaped problems whose runs are cut
      // into blocks: +6.3 % in the geometric mean (up to +33 %: 9472-byte runs in blocks of 1360 bytes, 4.0 TB/s,
      // in blocks of 1920, 5.3) with 128 bytes, +5.8 % with 64, +2.6 % with 32, +6.5 % with 256.
      if (cb > 1) c = std::min<int64_t>(t, (c + align_vecs - 1) / align_vecs * align_vecs);
      if ((cb - 1) * c >= max_run_vecs) continue;   // the rounding left the last block empty
      if (cb > cb_min && c < 16) break;   // keep at least 256 contiguous bytes per row of a tile
      const double f = (double)max_run_vecs * (double)(t / c) / (double)(cb * t);  // fraction of lanes with work
      if (f > best + 0.04) { best = f; *tc_out = c; *tr_out = t / c; }
    }
    return best;
  };
  int extra_blocks = 0;
  if (v == 16 && op.unroll == 1 && !unroll_fixed) {
    // Runs that leave many of 256 lanes idle (148 vectors: 42 % of the lanes busy).  Two ways out: rows cut into up
    // to 7 more column blocks than necessary, ending on 128-byte boundaries (7 blocks of 78 for 540 vectors, three
    // rows per tile: 90 %), or more vectors per thread, which pack more whole rows into a tile (148 vectors: 87 %
    // with four).  Column blocks come first where they keep 80 % of the lanes busy and no more than 4 points fewer
    // than the other way: measured on the 20 such ops among 1000 paper-shaped problems, +5.7 % in the geometric mean
    // (192-vector runs in blocks of 64, four rows a tile, against five whole rows with four vectors per thread:
    // 5.1 -> 6.1 TB/s; 333-vector runs, 93 % against 98 % of the lanes: -4.5 %, so those keep their whole rows).
    // (Destination-major order keeps one vector per thread in any case.)
    int64_t c, r2;
    const double whole = shape_of(1, 0, &c, &r2);
    if (whole < 0.8) {
      double by_unroll = whole;
      int u_best = 1;
      for (int u : {2, 4}) {
        const double f = shape_of(u, 0, &c, &r2);
        if (!op.dest_major && by_unroll < 0.8 && f > by_unroll + 0.04) { by_unroll = f; u_best = u; }
      }
      const double by_blocks = shape_of(1, 7, &c, &r2);
      if (by_blocks >= 0.8 && by_blocks + 0.04 >= by_unroll) extra_blocks = 7;
      else if (u_best != 1) op.unroll = u_best;
      else if (by_blocks > whole + 0.04) extra_blocks = 7;
    }
  }
  if (v != 16) op.unroll = 4;  // narrower vectors are instantiated for 4 per thread only
  int64_t tc, tr;
  shape_of(op.unroll, extra_blocks, &tc, &tr);
  op.tc = (int)tc;
  op.tr = (int)tr;
  {
    uint8_t sh = 0;
    magic_for((uint32_t)tc, &op.tc_magic, &sh);
    op.tc_shift = sh;
  }

  if (op.dest_major) {
    const int64_t tile_bytes = 256ll * op.unroll * v;
    op.chunk_tiles = 8;   // a power of two (the kernel shifts), at most 16 MiB of source
    while ((int64_t)op.chunk_tiles * 2 * tile_bytes <= (16ll << 20)) op.chunk_tiles *= 2;
  }
  uint64_t tiles = 0;
  bool uniform = true;
  op.boxes.reserve(hb.size());
  for (const auto& b : hb) {
    DevBox db{};
    db.src_off = b.soff * elem_size;
    db.dst_off = b.doff * elem_size;
    db.src_dev = b.src_dev;
    db.dst_first = b.dst_first;
    db.dst_count = b.dst_count;
    db.dst_dev0 = op.dst_list[(size_t)b.dst_first];
    int64_t run_vecs = b.len[ng - 1] * elem_size / v;
    int64_t rows = 1;
    for (int k = 0; k < op.n_outer; ++k) {
      int64_t l = b.len[keep[k]];
      rows *= l;
      if (l >= (1ll << 31)) return false;
      db.len[k] = (uint32_t)l;
      magic_for((uint32_t)l, &db.magic[k], &db.shift[k]);
    }
    if (rows >= (1ll << 31) || run_vecs >= (1ll << 31)) return false;
    db.run_vecs = (uint32_t)run_vecs;
    db.rows = (uint32_t)rows;
    int64_t cbs = (run_vecs + tc - 1) / tc, rbs = (rows + tr - 1) / tr;
    if (cbs * rbs >= (1ll << 31)) return false;
    db.col_blocks = (uint32_t)cbs;
    magic_for(db.col_blocks, &db.cb_magic, &db.cb_shift);
    db.n_tiles = (uint32_t)(cbs * rbs);
    db.tile_first = (uint32_t)tiles;
    tiles += db.n_tiles;
    if (tiles >= (1ull << 31)) return false;
    if (!op.boxes.empty() && db.n_tiles != op.boxes.front().n_tiles) uniform = false;
    int64_t box_bytes = rows * run_vecs * v;
    op.bytes_read += box_bytes;
    op.bytes_written += box_bytes * db.dst_count;
    op.boxes.push_back(db);
  }
  // destination-major order: every tile of the op once per destination
  op.src_tiles = (uint32_t)tiles;
  op.dm_count = op.dest_major ? (uint32_t)op.boxes.front().dst_count : 1u;
  if (op.dest_major) {
    const bool fixed = opt.dm_fanout == 1 || opt.dm_fanout == 2;
    op.dm_fanout = fixed ? (uint32_t)opt.dm_fanout : (op.dm_count <= 8 ? 2u : 1u);
    op.dm_groups = (op.dm_count + op.dm_fanout - 1) / op.dm_fanout;
  }
  if (tiles * op.dm_groups >= (1ull << 31)) return false;
  if (op.dest_major) {
    uint8_t sh = 0;
    magic_for(op.dm_groups, &op.dm_magic, &sh);   // (the kernel does not use it when dm_groups is 1)
    op.dm_shift = sh;
  }
  op.n_tiles = (uint32_t)(tiles * op.dm_groups);
  op.tiles_per_box = (uniform && !op.boxes.empty()) ? op.boxes.front().n_tiles : 0;
  if (op.sib_count > 1 && (op.tiles_per_box == 0 || op.unroll != 1 || op.boxes.size() % op.sib_count))
    op.sib_count = 1;   // (the kernel finds the box of a tile without a descriptor: one box shape)
  if (op.sib_count > 1 && op.tr == 1) {   // runs of several tiles: a power of two of them, every box the same
    const uint32_t cb = op.boxes.front().col_blocks;
    for (const auto& b : op.boxes)
      if (b.col_blocks != cb) op.sib_count = 1;
    if (cb & (cb - 1)) op.sib_count = 1;
    while (op.sib_count > 1 && (1u << op.sib_inner_log2) < cb) ++op.sib_inner_log2;
  }
  if (op.sib_count > 1) {
    uint8_t sh = 0;
    magic_for(op.sib_count, &op.sib_magic, &sh);
    op.sib_shift = sh;
  }
  if (op.tiles_per_box > 1) {
    uint8_t sh = 0;
    magic_for(op.tiles_per_box, &op.tpb_magic, &sh);
    op.tpb_shift = sh;
  }
  *out = std::move(op);
  return true;
}
}  // namespace

}  // namespace redist

// ---------------------------------------------------------------------------------------------------
namespace redist {
namespace {
bool is_pow2(int64_t v) { return v > 0 && (v & (v - 1)) == 0; }
int log2_of(int64_t v) { int l = 0; while ((1ll << l) < v) ++l; return l; }
}  // namespace

namespace {
bool build_row_op_last_dim(int ndev, int rank, int elem_size, const std::vector<int64_t>& cs,
                           const std::vector<int64_t>& os, const std::vector<int64_t>& cd,
                           const std::vector<int64_t>& od, const BuildOptions& opt, RowOp* out);
}  // namespace

bool fold_untouched_last_dims(int ndev, int rank, std::vector<int64_t>* cs_io, std::vector<int64_t>* os_io,
                              std::vector<int64_t>* cd_io, std::vector<int64_t>* od_io) {
  const int r = rank;
  std::vector<int64_t>&cs = *cs_io, &os = *os_io, &cd = *cd_io, &od = *od_io;
  for (int folded = 0; r >= 2 && cs[(size_t)r - 1] == cd[(size_t)r - 1]; ++folded) {
    if (folded == r - 1) return false;
    const int64_t c = cs[(size_t)r - 1];
    auto fold = [&](std::vector<int64_t>& shape, std::vector<int64_t>& offs) {
      for (int d = 0; d < ndev; ++d) {
        int64_t* o = offs.data() + (size_t)d * r;
        const int64_t which = o[r - 1] / c, merged = o[r - 2] * c;
        for (int t = r - 2; t >= 1; --t) o[t] = o[t - 1];
        o[0] = which;
        o[r - 1] = merged;
      }
      const int64_t merged = shape[(size_t)r - 2] * c;
      for (int t = r - 2; t >= 1; --t) shape[(size_t)t] = shape[(size_t)t - 1];
      shape[0] = 1;
      shape[(size_t)r - 1] = merged;
    };
    fold(cs, os);
    fold(cd, od);
  }
  return true;
}

bool build_row_op(int ndev, int rank, int elem_size, const std::vector<int64_t>& shape_s,
                  const std::vector<int64_t>& offs_s, const std::vector<int64_t>& shape_d,
                  const std::vector<int64_t>& offs_d, const BuildOptions& opt, RowOp* out) {
  if (!opt.lds_staging) return false;  // the caller asked for the generic body
  // A last dim with the same tile extent c on both sides is not touched by the step: the rows that matter are
  // those of the dim before it, c times as long (a step on a dim of 4 in front of a last dim of 8 four-byte
  // elements moves 32-byte pieces).  The tables are rewritten to say so without changing any shard's memory
  // layout: the last dim folds into the one before it (tile extent and offsets times c), and which of its tiles a
  // device holds, which source and destination of a piece must agree on, becomes a new leading dim of extent 1.
  const int r = rank;
  std::vector<int64_t> cs = shape_s, os = offs_s, cd = shape_d, od = offs_d;
  if (!fold_untouched_last_dims(ndev, r, &cs, &os, &cd, &od)) return false;   // nothing but untouched dims
  return build_row_op_last_dim(ndev, r, elem_size, cs, os, cd, od, opt, out);
}

namespace {
bool build_row_op_last_dim_impl(int ndev, int rank, int elem_size, const std::vector<int64_t>& cs,
                                const std::vector<int64_t>& os, const std::vector<int64_t>& cd,
                                const std::vector<int64_t>& od, const BuildOptions& opt, int64_t cut_rows, RowOp* out);

// The general form learns its rows per tile late (from the vector widths the offsets allow), so its boxes are cut
// for destination order (see below) in a second pass that knows them; the result counts when it is the same form.
bool build_row_op_last_dim(int ndev, int rank, int elem_size, const std::vector<int64_t>& cs,
                           const std::vector<int64_t>& os, const std::vector<int64_t>& cd,
                           const std::vector<int64_t>& od, const BuildOptions& opt, RowOp* out) {
  if (!build_row_op_last_dim_impl(ndev, rank, elem_size, cs, os, cd, od, opt, 0, out)) return false;
  if (out->general && !out->span && !out->dest_major && opt.row_dst_order) {
    RowOp cut;
    if (build_row_op_last_dim_impl(ndev, rank, elem_size, cs, os, cd, od, opt, (int64_t)out->rpt, &cut) && cut.general &&
        !cut.span && !cut.dest_major && cut.rpt == out->rpt && cut.vn == out->vn && cut.vw == out->vw &&
        cut.boxes.size() != out->boxes.size())
      *out = std::move(cut);
  }
  return true;
}

bool build_row_op_last_dim_impl(int ndev, int rank, int elem_size, const std::vector<int64_t>& cs,
                                const std::vector<int64_t>& os, const std::vector<int64_t>& cd,
                                const std::vector<int64_t>& od, const BuildOptions& opt, int64_t cut_rows, RowOp* out) {
  const int r = rank;
  if (cs[r - 1] == cd[r - 1]) return false;  // last dim untouched: runs are whole rows or longer
  RowOp op;
  op.dir = cd[r - 1] > cs[r - 1] ? 0 : 1;
  // wide side w, narrow side n
  const std::vector<int64_t>& cw = op.dir == 0 ? cd : cs;
  const std::vector<int64_t>& ow = op.dir == 0 ? od : os;
  const std::vector<int64_t>& cn = op.dir == 0 ? cs : cd;
  const std::vector<int64_t>& on = op.dir == 0 ? os : od;
  if (cw[r - 1] % cn[r - 1]) return false;
  const int64_t W = cw[r - 1] * elem_size, N = cn[r - 1] * elem_size;
  // runs long enough for the generic kernel, unless they start and end in the middle of cache lines
  // (measured on 592- and 720-byte runs: 4.1 TB/s generic, 5.4 TB/s staged)
  if (N >= 512 && (N % 128 == 0 || N > 4096)) return false;
  op.w_bytes = (uint32_t)W;
  op.n_bytes = (uint32_t)N;
  op.n_pieces = (int)(W / N);
  // (power-of-two pieces narrower than a vector stay with this form's narrow vectors: the span form measured
  //  slower on them, 3.2-4.0 against 4.5-5.5 TB/s on 4-byte pieces of 256-byte rows)
  op.general = !(is_pow2(W) && is_pow2(N) && W >= 16 && W <= 4096);
  if (!op.general) {
    op.w_log2 = log2_of(W);
    op.n_log2 = log2_of(N);
    op.vn = (int)std::min<int64_t>(16, N);
    int64_t R = kRowTileBytes / W;
    // (256 rows at most, one per thread of the offsets phase; rows of 16 and 32 bytes take the kernel variant
    //  with tables for 1024 rows, so that their tiles are 16 KiB too: measured 2.9-3.9 TB/s with 4 and 8 KiB tiles)
    op.r_log2 = log2_of(std::min<int64_t>(W <= 32 ? 1024 : 256, std::max<int64_t>(4, R)));
  } else {
    if (W > 8192 || W < 8) return false;
    op.vn = pow2_floor_gcd(N, 16);                   // refined below by offsets and strides
  }

  // outer dims = all but the last; strides in bytes on both sides
  const int no = r - 1;
  std::vector<int64_t> ws(no), ns(no);
  {
    int64_t a = W, b = N;
    for (int t = no - 1; t >= 0; --t) { ws[t] = a; ns[t] = b; a *= cw[t]; b *= cn[t]; }
  }
  std::map<std::vector<int64_t>, std::vector<int>> wide_groups, narrow_holders;
  std::vector<std::vector<int64_t>> order;
  for (int d = 0; d < ndev; ++d) {
    std::vector<int64_t> key(ow.begin() + (size_t)d * r, ow.begin() + (size_t)(d + 1) * r);
    auto& v = wide_groups[key];
    if (v.empty()) order.push_back(key);
    v.push_back(d);
    narrow_holders[std::vector<int64_t>(on.begin() + (size_t)d * r, on.begin() + (size_t)(d + 1) * r)].push_back(d);
  }
  op.narrow_count = op.dir == 0 ? 1 : (int)narrow_holders.begin()->second.size();
  if ((int64_t)op.n_pieces * op.narrow_count > kRowMaxPtrs) return false;
  // Pieces of 256 and 384 bytes (whole 128-byte lines): the generic kernel is as good or better (16 ops among 1000
  // paper-shaped problems: +5 % in the geometric mean, -4 % ... +15 %), except where a scatter writes every piece to
  // several shards, which the staged destination-major order serves better (three ops: generic 7-12 % slower).
  if (N >= 256 && N % 128 == 0 && !(op.dir == 1 && op.narrow_count > 1)) return false;

  // Destination-major order (see RowOp) on meshes whose shard pointers travel as kernel arguments: ops of 32 MiB
  // and more that write every tile to the same number m > 1 of shards (every form but the power-of-two one with
  // tiles of 1024 rows).
  bool dm_forced = false;
  {
    const int64_t dm_min_bytes = std::max<int64_t>(0, opt.dest_major_min_bytes);
    dm_forced = dm_min_bytes == 0;
    int64_t m = op.dir == 1 ? op.narrow_count : (int64_t)wide_groups.begin()->second.size();
    bool same = m > 1;
    for (const auto& kv : wide_groups) same = same && (op.dir == 1 || (int64_t)kv.second.size() == m);
    int64_t wide_bytes = (int64_t)wide_groups.size() * elem_size;
    for (int t = 0; t < r; ++t) wide_bytes *= cw[t];
    op.dest_major = same && (op.general || op.r_log2 <= 8) && ndev <= 128 && wide_bytes >= dm_min_bytes &&
                    opt.dest_major;
    op.dm_count = op.dest_major ? (uint32_t)m : 1u;
  }
  // 128-byte pieces in the usual order go through the generic kernel as well (15 ops among 1000 paper-shaped
  // problems: +7 % in the geometric mean, none beyond -2 %); in destination-major order the staged form stays (8 ops:
  // -15 % ... +14 % either way).
  if (N == 128 && !op.dest_major) return false;
  struct HostRow { int64_t woff; int wide_first, wide_count, piece_first; std::vector<int64_t> len; };
  std::vector<HostRow> hb;
  for (const auto& key : order) {
    const std::vector<int>& members = wide_groups[key];
    int wide_first = (int)op.dev_list.size();
    op.dev_list.insert(op.dev_list.end(), members.begin(), members.end());
    std::vector<std::vector<Seg>> segs(no);
    for (int t = 0; t < no; ++t) {
      int64_t o = key[t], end = o + cw[t];
      for (int64_t k = o / cn[t]; k * cn[t] < end; ++k) {
        int64_t lo = std::max(o, k * cn[t]), hi = std::min(end, (k + 1) * cn[t]);
        segs[t].push_back(Seg{lo - o, hi - lo, lo - k * cn[t], k});  // dst_start := wide, src_start := narrow
      }
    }
    std::vector<size_t> idx(no, 0);
    while (true) {
      HostRow b;
      b.woff = 0;
      b.wide_first = wide_first;
      b.wide_count = (int)members.size();
      b.piece_first = (int)op.pieces.size();
      int64_t noff = 0;
      std::vector<int64_t> nkey(r);
      for (int t = 0; t < no; ++t) {
        const Seg& sg = segs[t][idx[t]];
        b.woff += sg.dst_start * ws[t];
        noff += sg.src_start * ns[t];
        b.len.push_back(sg.len);
        nkey[t] = sg.src_tile * cn[t];
      }
      for (int k = 0; k < op.n_pieces; ++k) {
        nkey[r - 1] = key[r - 1] + (int64_t)k * cn[r - 1];
        auto it = narrow_holders.find(nkey);
        if (it == narrow_holders.end()) return false;
        DevPiece pc{};
        pc.narrow_off = noff;
        pc.dev_first = (int)op.dev_list.size();
        if (op.dir == 0) {
          // gather: one source replica; prefer one that is also a destination -- except in destination-major
          // order, where the lowest-numbered holder serves everyone and is read front to back
          int src = it->second.front();
          for (int h : it->second)
            if (!op.dest_major && std::find(members.begin(), members.end(), h) != members.end()) { src = h; break; }
          op.dev_list.push_back(src);
        } else {
          if ((int)it->second.size() != op.narrow_count) return false;
          op.dev_list.insert(op.dev_list.end(), it->second.begin(), it->second.end());
        }
        op.pieces.push_back(pc);
      }
      hb.push_back(std::move(b));
      int t = no - 1;
      while (t >= 0 && ++idx[t] == segs[t].size()) idx[t--] = 0;
      if (t < 0) break;
    }
  }
  // Destination order (ops in the usual order; power-of-two form and row-by-row general form).  A box is a range of every outer dim; its tiles
  // go row-major through it, so with several boxes per destination shard -- the pieces of different source shards --
  // each box leaves gaps in the destination that another box fills later, and the window of addresses being
  // written is sparse.  So the boxes are cut along their leading dims into parts that are one contiguous stretch of
  // the destination each (whole tiles: else the boxes stay), and the parts sorted by where they write: the op then
  // fills each destination shard front to back (what the generic kernel's sibling boxes do for runs, see
  // CopyOp::sib_count).  Measured on the attention pairs: 8 KiB stretches of eight sources, 4.4 -> 5.6 TB/s; cutting
  // further, into parts that are several stretches, lost 4 %; parts that come out in the order they had are not cut
  // (more descriptors for nothing: -3 %).
  if (!op.dest_major && (!op.general || cut_rows > 0) && opt.row_dst_order && !hb.empty() && no >= 2) {
    const int64_t Rt = op.general ? cut_rows : 1ll << op.r_log2;
    const std::vector<int64_t>& dstride = op.dir == 0 ? ws : ns;   // the side written
    int t_split = 0;                                                // dims [0, t_split) are cut into single indices
    bool whole = true;
    int64_t n_parts = 0;
    for (const auto& b : hb) {
      int t = no - 1;
      while (t > 0 && dstride[(size_t)t - 1] == dstride[(size_t)t] * b.len[(size_t)t]) --t;
      t_split = std::max(t_split, t);
    }
    for (const auto& b : hb) {
      int64_t rem = 1, lead = 1;
      for (int u = t_split; u < no; ++u) rem *= b.len[(size_t)u];
      for (int u = 0; u < t_split; ++u) lead *= b.len[(size_t)u];
      whole = whole && rem % Rt == 0;
      n_parts += lead;
    }
    // (every part carries its own piece descriptors: at most 4 MiB of them)
    if (t_split > 0 && whole && n_parts <= 65536 && n_parts * op.n_pieces <= 262144 && n_parts > (int64_t)hb.size()) {
      struct Part { HostRow row; int64_t noff; size_t parent, seq; };
      std::vector<Part> parts;
      for (size_t q = 0; q < hb.size(); ++q) {
        const HostRow& b = hb[q];
        std::vector<int64_t> idx((size_t)t_split, 0);
        for (size_t seq = 0;; ++seq) {
          Part pt{b, op.pieces[(size_t)b.piece_first].narrow_off, q, seq};
          for (int u = 0; u < t_split; ++u) {
            pt.row.woff += idx[(size_t)u] * ws[(size_t)u];
            pt.noff += idx[(size_t)u] * ns[(size_t)u];
            pt.row.len[(size_t)u] = 1;
          }
          parts.push_back(std::move(pt));
          int u = t_split - 1;
          while (u >= 0 && ++idx[(size_t)u] == b.len[(size_t)u]) idx[(size_t)u--] = 0;
          if (u < 0) break;
        }
      }
      auto key_of = [&](const Part& pt) {   // first shard written, offset there
        if (op.dir == 0) return std::make_pair(op.dev_list[(size_t)pt.row.wide_first], pt.row.woff);
        return std::make_pair(op.dev_list[(size_t)op.pieces[(size_t)pt.row.piece_first].dev_first], pt.noff);
      };
      std::stable_sort(parts.begin(), parts.end(), [&](const Part& x, const Part& y) { return key_of(x) < key_of(y); });
      bool interleaved = false;   // does any box's sequence of parts get interrupted?
      for (size_t q = 1; q < parts.size() && !interleaved; ++q)
        interleaved = parts[q].seq != 0 && (parts[q - 1].parent != parts[q].parent || parts[q - 1].seq + 1 != parts[q].seq);
      if (interleaved) {
        std::vector<DevPiece> part_pieces;
        std::vector<HostRow> rows;
        for (auto& pt : parts) {
          const int64_t dn = pt.noff - op.pieces[(size_t)pt.row.piece_first].narrow_off;
          const size_t first = part_pieces.size();
          for (int k = 0; k < op.n_pieces; ++k) {
            DevPiece pc = op.pieces[(size_t)pt.row.piece_first + (size_t)k];
            pc.narrow_off += dn;
            part_pieces.push_back(pc);
          }
          pt.row.piece_first = (int)first;
          rows.push_back(std::move(pt.row));
        }
        op.pieces = std::move(part_pieces);
        hb = std::move(rows);
      }
    }
  }
  if (op.dest_major) {   // boxes in source order: chunks of the op are then dense stretches of the shards read
    auto key_of = [&](const HostRow& b) {
      if (op.dir == 1) return std::make_pair(op.dev_list[(size_t)b.wide_first], b.woff);
      const DevPiece& pc = op.pieces[(size_t)b.piece_first];
      return std::make_pair(op.dev_list[(size_t)pc.dev_first], pc.narrow_off);
    };
    std::stable_sort(hb.begin(), hb.end(), [&](const HostRow& x, const HostRow& y) { return key_of(x) < key_of(y); });
  }
  // drop outer dims of extent 1 everywhere; merge neighbours that every box covers as one contiguous
  // range on both sides (the inner one whole), so that rows stay contiguous for as long as possible
  std::vector<int64_t> kws, kns;               // strides of the kept dims
  std::vector<std::vector<int64_t>> klen(hb.size());
  for (int t = 0; t < no; ++t) {
    bool all_one = true;
    for (const auto& b : hb) all_one = all_one && b.len[t] == 1;
    if (all_one) continue;
    bool merged = false;
    if (!kws.empty()) {
      // dim t continues the previous kept dim when stepping the previous one by 1 equals stepping t by its full length
      bool same = true;
      const int64_t l0 = hb.front().len[t];
      for (const auto& b : hb) same = same && b.len[t] == l0;
      if (same && kws.back() == ws[t] * l0 && kns.back() == ns[t] * l0) {
        for (size_t q = 0; q < hb.size(); ++q) klen[q].back() *= l0;
        kws.back() = ws[t];
        kns.back() = ns[t];
        merged = true;
      }
    }
    if (!merged) {
      kws.push_back(ws[t]);
      kns.push_back(ns[t]);
      for (size_t q = 0; q < hb.size(); ++q) klen[q].push_back(hb[q].len[t]);
    }
  }
  op.n_outer = (int)kws.size();
  if (op.n_outer > kMaxOuter) return false;
  for (int k = 0; k < kMaxOuter; ++k) { op.wstride[k] = 0; op.nstride[k] = 0; }
  for (int k = 0; k < op.n_outer; ++k) { op.wstride[k] = kws[k]; op.nstride[k] = kns[k]; }
  if (op.dest_major && !dm_forced) {
    // every box one contiguous stretch of the shard it reads (rows of a box that lie apart would share cache sets)
    const std::vector<int64_t>& st = op.dir == 1 ? kws : kns;
    for (size_t q = 0; q < hb.size() && op.dest_major; ++q) {
      int64_t cnt = op.dir == 1 ? W : N;
      for (int k = op.n_outer - 1; k >= 0; --k) {
        if (klen[q][(size_t)k] > 1 && st[(size_t)k] != cnt) op.dest_major = false;
        cnt *= klen[q][(size_t)k];
      }
    }
    if (!op.dest_major) op.dm_count = 1;   // the usual order then; box order and source replicas may stay as they are
  }
  if (!op.general) {
    // alignment: wide side moves 16-byte vectors, narrow side vn-byte vectors
    for (int k = 0; k < op.n_outer; ++k)
      if (op.wstride[k] % 16 || op.nstride[k] % op.vn) return false;
    for (const auto& b : hb)
      if (b.woff % 16) return false;
    for (const auto& pc : op.pieces)
      if (pc.narrow_off % op.vn) return false;
  } else {
    // narrow side: the widest vector every piece, offset and stride allows; wide side: 16 bytes when
    // the wide rows, offsets and strides allow, else the narrow width
    int v = op.vn, vw = pow2_floor_gcd(W, 16);
    for (int k = 0; k < op.n_outer; ++k) { vw = pow2_floor_gcd(op.wstride[k], vw); v = pow2_floor_gcd(op.nstride[k], v); }
    for (const auto& b : hb) vw = pow2_floor_gcd(b.woff, vw);
    for (const auto& pc : op.pieces) v = pow2_floor_gcd(pc.narrow_off, v);
    if (vw != 16) { v = std::min(v, vw); vw = v; }
    op.vn = v;
    op.vw = vw;
    // Span form: when a side cannot move 16-byte vectors row by row.  Rows that are contiguous on both sides
    // (the innermost outer dim steps by exactly one row; else every row on its own) form chunks; a tile is
    // made of virtual chunks -- whole chunks, or stretches of rpt rows of a long one -- each of them one
    // contiguous span per side, which 16-byte aligned blocks cover regardless of where rows start.
    const bool contiguous_rows = op.n_outer > 0 && op.wstride[op.n_outer - 1] == W && op.nstride[op.n_outer - 1] == N;
    // Not for scatters that write every piece to several shards: measured on MI355X, those run 15-20 % faster
    // with the row-by-row form's many narrow stores than with bursts of 16-byte ones (gathers with replicated
    // destinations: no clear difference).
    const bool replicating = op.dir == 1 && op.narrow_count > 1;
    // Nor for scatters whose wide side moves whole vectors row by row and whose pieces are multiples of 8 bytes:
    // the row-by-row form is as fast there (measured 5.9 against 5.6 TB/s).
    const bool row_by_row_is_fine = op.dir == 1 && vw == 16 && v == 8;
    if (v < 16 && !replicating && !row_by_row_is_fine && opt.span_form) {
      int64_t cr_min = 1, cr_max = 1;
      if (contiguous_rows) {
        cr_min = INT64_MAX;
        cr_max = 0;
        for (const auto& l : klen) { cr_min = std::min(cr_min, l.back()); cr_max = std::max(cr_max, l.back()); }
      }
      const int64_t R = std::max<int64_t>(1, kRowTileBytes / W);       // rows of a virtual chunk, at most
      const int64_t vrows = std::min(R, cr_max);
      const int64_t cbw = (vrows * W + 15) / 16 + 1, cbn = (vrows * N + 15) / 16 + 1;   // blocks per span, at most
      int64_t m = std::min<int64_t>(kRowMaxChunks, (kRowTileBytes + 32) / (16 * cbw));
      m = std::min<int64_t>(m, kRowMaxPtrs / ((int64_t)op.n_pieces * op.narrow_count));
      // worth it when tiles come out large and a chunk's piece span is more than its two edge blocks
      const int64_t small = std::min(R, cr_min);
      if (m >= 1 && m * small * W >= 8192 && small * N >= 48) {
        op.span = true;
        op.gran = v;
        op.chunk_dims = contiguous_rows ? op.n_outer - 1 : op.n_outer;
        op.wide_shard_bytes = elem_size;
        op.narrow_shard_bytes = elem_size;
        for (int t = 0; t < r; ++t) { op.wide_shard_bytes *= cw[t]; op.narrow_shard_bytes *= cn[t]; }
        op.rpt = (uint32_t)R;
        op.mct = (uint32_t)m;
        op.slot = (uint32_t)(16 * cbw);
        op.cbw = (uint32_t)cbw;
        op.nbm = (uint32_t)cbn;
        op.cpn = (uint32_t)(N / v);                          // granules per piece row
        uint8_t sh = 0;
        magic_for(op.cpn, &op.cpn_magic, &sh); op.cpn_shift = sh;
        magic_for(op.nbm, &op.nbm_magic, &sh); op.nbm_shift = sh;
        magic_for(op.cbw, &op.cbw_magic, &sh); op.cbw_shift = sh;
      }
    }
    if (op.span) {
    } else {
      // staged rows are padded to a 16-byte multiple plus 16, so that consecutive rows start 4 banks apart
      op.pitch = (uint32_t)((W + 15) / 16 * 16 + 16);
      int64_t R = std::min<int64_t>(256, kRowTileBytes / op.pitch);
      if (R < 2) return false;
      // Any number of rows per tile (a division more per narrow vector): a power of two left 24-40 % of the staging
      // area empty for most row lengths (160-byte rows: 64 of 93 rows).  But tile boundaries must fall on 128-byte
      // (else 64-byte) boundaries of both sides' stretches -- 43 rows of 180-byte pieces instead of 32 lost 30 %,
      // 48 rows of 144-byte pieces instead of 32 gained 8 % --, and tiles should not straddle the ends of short
      // innermost ranges (64 rows a range: tiles of 96 rows lost 5 % against 64).  So the number of rows is the
      // largest multiple of the alignment that fills 5/8 of the area at least and, for innermost ranges under four
      // tiles, divides the range or is a multiple of it; else the largest power of two as before (unless that straddles
      // too and an aligned number exists).  Measured on the 35
      // such ops among 300 paper-shaped problems: +2.3 % in the geometric mean (-10 % ... +10 %).  Destination-major
      // ops keep the power of two (nine ops: -6 % ... 0).
      {
        int64_t inner = 0;   // rows of the innermost range, when every box has the same
        if (op.n_outer > 0) {
          inner = klen.front().back();
          for (const auto& l : klen)
            if (l.back() != inner) inner = 0;
        }
        auto clean = [&](int64_t q) { return inner == 0 || inner >= 4 * q || inner % q == 0 || q % inner == 0; };
        int64_t pow2 = 1, chosen = 0, aligned = 0;
        while (pow2 * 2 <= R) pow2 *= 2;
        for (int64_t line : {128, 64}) {
          if (op.dest_major) break;
          const int64_t al = std::max(line / std::gcd<int64_t>(W, line), line / std::gcd<int64_t>(N, line));
          for (int64_t q = R / al * al; q > 0 && q * 8 >= R * 5; q -= al) {
            if (aligned == 0) aligned = q;
            if (clean(q)) { chosen = q; break; }
          }
          if (chosen) break;
        }
        if (chosen == 0) chosen = (aligned == 0 || clean(pow2)) ? pow2 : aligned;
        R = chosen;
      }
      op.rpt = (uint32_t)R;
      {
        uint8_t sh = 0;
        magic_for(op.rpt, &op.rpt_magic, &sh);
        op.rpt_shift = sh;
      }
      op.r_log2 = 0;   // (floor of log2, for the record: nothing computes with it in this form)
      while ((2ll << op.r_log2) <= R) ++op.r_log2;
      op.cpn = (uint32_t)(N / v);
      op.wpr = (uint32_t)(W / vw);
      uint8_t sh = 0;
      magic_for(op.cpn, &op.cpn_magic, &sh); op.cpn_shift = sh;
      magic_for(op.wpr, &op.wpr_magic, &sh); op.wpr_shift = sh;
    }
  }

  op.max_grid = std::max(1u, std::min(opt.max_grid, 16777215u));
  // Destination-major order stages a tile once per receiving shard.  That pays where staging is cheap next to the
  // memory traffic; the row-by-row general form with vectors narrower than 8 bytes on the narrow side, or narrower
  // than 16 on the wide side, is bound by the instructions it issues per byte and lost a third of its rate in this
  // order (measured on 360-byte rows of 180-byte pieces, 4-byte vectors: 5.0-5.5 -> 3.3-3.5 TB/s), while wider
  // vectors and the span form gained 10-40 % on most ops.
  if (op.dest_major && !dm_forced && op.general && !op.span && !(op.vw == 16 && op.vn >= 8)) {
    op.dest_major = false;
    op.dm_count = 1;
  }
  const int64_t Rr = op.span || op.general ? (int64_t)op.rpt : (1ll << op.r_log2);
  uint64_t tiles = 0;
  bool uniform = true;
  for (size_t q = 0; q < hb.size(); ++q) {
    const auto& b = hb[q];
    DevRowBox db{};
    db.wide_off = b.woff;
    db.wide_first = b.wide_first;
    db.wide_count = b.wide_count;
    db.piece_first = b.piece_first;
    int64_t rows = 1;
    for (int k = 0; k < op.n_outer; ++k) {
      int64_t l = klen[q][k];
      rows *= l;
      if (l >= (1ll << 31)) return false;
      db.len[k] = (uint32_t)l;
      magic_for((uint32_t)l, &db.magic[k], &db.shift[k]);
    }
    if (rows >= (1ll << 31)) return false;
    db.rows = (uint32_t)rows;
    if (op.span) {
      const int64_t cr = op.chunk_dims < op.n_outer ? klen[q].back() : 1;
      // A chunk longer than a tile is cut into stretches of equal length -- or, where that many rows fit, of a
      // number of rows that makes every cut fall on a 128-byte (else 64-byte) boundary of both sides' spans.
      int64_t vrows = (cr + (cr + Rr - 1) / Rr - 1) / ((cr + Rr - 1) / Rr);
      if (cr > Rr) {
        for (int64_t line : {128, 64}) {
          const int64_t al = std::max(line / std::gcd<int64_t>(W, line), line / std::gcd<int64_t>(N, line));
          // (smaller tiles, or one more short stretch per chunk, cost more than cuts inside lines)
          const int64_t q = Rr / al * al;
          if (q * 8 >= Rr * 7 && ((cr + q - 1) / q) * 20 <= ((cr + Rr - 1) / Rr) * 21) { vrows = q; break; }
        }
      }
      const int64_t tpc = (cr + vrows - 1) / vrows;
      const int64_t nv = (rows / cr) * tpc;           // virtual chunks of the box
      if (nv >= (1ll << 31)) return false;
      db.chunk_rows = (uint32_t)cr;
      db.tpc = (uint32_t)tpc;
      magic_for(db.tpc, &db.tpc_magic, &db.tpc_shift);
      db.n_vchunks = (uint32_t)nv;
      db.vrows = (uint32_t)vrows;
      db.n_tiles = (uint32_t)((nv + op.mct - 1) / op.mct);
    } else {
      db.n_tiles = (uint32_t)((rows + Rr - 1) / Rr);
    }
    db.tile_first = (uint32_t)tiles;
    tiles += db.n_tiles;
    if (tiles >= (1ull << 31)) return false;
    if (!op.boxes.empty() && db.n_tiles != op.boxes.front().n_tiles) uniform = false;
    op.boxes.push_back(db);
    op.bytes_read += rows * W;
    op.bytes_written += rows * W * (op.dir == 0 ? db.wide_count : op.narrow_count);
  }
  op.src_tiles = (uint32_t)tiles;
  {
    // rows that follow each other in memory on a side share a stretch (the innermost outer dim steps by one row)
    const bool wc = op.n_outer > 0 && op.wstride[op.n_outer - 1] == W, ncg = op.n_outer > 0 && op.nstride[op.n_outer - 1] == N;
    op.min_stretch = INT64_MAX;
    for (size_t q = 0; q < hb.size(); ++q) {
      const int64_t inner = op.n_outer > 0 ? std::min<int64_t>(klen[q].back(), Rr) : 1;
      op.min_stretch = std::min(op.min_stretch, std::min(W * (wc ? inner : 1), N * (ncg ? inner : 1)));
    }
  }
  if (op.dest_major) {
    const bool fixed = opt.dm_fanout == 1 || opt.dm_fanout == 2;
    op.dm_fanout = fixed ? (uint32_t)opt.dm_fanout : (op.dm_count <= 8 ? 2u : 1u);
    op.dm_groups = (op.dm_count + op.dm_fanout - 1) / op.dm_fanout;
  }
  if (tiles * op.dm_groups >= (1ull << 31)) return false;
  op.n_tiles = (uint32_t)(tiles * op.dm_groups);
  if (op.dest_major) {
    op.chunk_tiles = (uint32_t)((16ll << 20) / kRowTileBytes);   // 16 MiB of source, a power of two
    uint8_t sh = 0;
    magic_for(op.dm_groups, &op.dm_magic, &sh);   // (not used by the kernel when there is one group)
    op.dm_shift = sh;
  }
  op.tiles_per_box = (uniform && !op.boxes.empty()) ? op.boxes.front().n_tiles : 0;
  if (op.tiles_per_box > 1) {
    uint8_t sh = 0;
    magic_for(op.tiles_per_box, &op.tpb_magic, &sh);
    op.tpb_shift = sh;
  }
  op.enabled = true;
  *out = std::move(op);
  return true;
}

}  // namespace

}  // namespace redist
