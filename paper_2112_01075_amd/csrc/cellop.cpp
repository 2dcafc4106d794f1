// Cell-complete description of a redistribution step (see DevCellBox in copyop.hpp): the innermost dims whose tiling
// changes are taken whole on both sides, so that a workgroup reads one contiguous stretch of every source tile of a
// cell and writes one contiguous stretch of every destination tile.
#include <algorithm>
#include <map>
#include <numeric>

#include "copyop.hpp"

namespace redist {

namespace {

int pow2_gcd(int64_t a, int v) {  // largest power of two <= v dividing a
  while (v > 1 && (a % v)) v >>= 1;
  return v;
}

struct Candidate {
  int n_cell = 0;
  int64_t rows = 0, stretch = 0;
};

struct HostCellBox {
  int64_t src_off = 0, dst_off = 0;
  int32_t src_first = 0, dst_first = 0;
  std::vector<int64_t> len;   // extents of the dims in front of the cell dims, the last of them the row dim
};

}  // namespace

bool build_cell_op(int ndev, int rank, int elem_size, const std::vector<int64_t>& shape_s,
                   const std::vector<int64_t>& offs_s, const std::vector<int64_t>& shape_d,
                   const std::vector<int64_t>& offs_d, const BuildOptions& opt, const OtherBody& other, CellOp* out) {
  if (!opt.lds_staging || opt.cell_form == 0 || ndev > 128) return false;
  const int r = rank;
  std::vector<int64_t> cs = shape_s, os = offs_s, cd = shape_d, od = offs_d;
  if (!fold_untouched_last_dims(ndev, r, &cs, &os, &cd, &od)) return false;
  if (cs[(size_t)r - 1] == cd[(size_t)r - 1]) return false;
  const int64_t B = elem_size;
  const int gran = pow2_gcd(std::min(cs[(size_t)r - 1], cd[(size_t)r - 1]) * B, 16);
  if (gran < 4) return false;

  // global extents, from the tables
  std::vector<int64_t> G((size_t)r, 0);
  for (int d = 0; d < ndev; ++d)
    for (int t = 0; t < r; ++t) {
      G[(size_t)t] = std::max(G[(size_t)t], os[(size_t)d * r + t] + cs[(size_t)t]);
      G[(size_t)t] = std::max(G[(size_t)t], od[(size_t)d * r + t] + cd[(size_t)t]);
    }

  // How many dims form the cell: the choice that gives the longest stretches (fewest dims among equals).
  Candidate best;
  {
    int64_t cell_bytes = B, src_row = B, dst_row = B, ps = 1, pd = 1;
    for (int nc = 1; nc <= kMaxCellDims && nc <= r; ++nc) {
      const int t = r - nc;
      const int64_t a = cs[(size_t)t], b = cd[(size_t)t], e = std::max(a, b);
      if (e % std::min(a, b) || G[(size_t)t] % e) break;   // tilings must be nested, cells whole
      cell_bytes *= e;
      src_row *= a;
      dst_row *= b;
      ps *= std::max<int64_t>(1, b / a);
      pd *= std::max<int64_t>(1, a / b);
      if (cell_bytes > kCellTileBytes || ps > kCellMaxParts || pd > kCellMaxParts) break;
      const int64_t row_limit = t > 0 ? std::min(cs[(size_t)t - 1], cd[(size_t)t - 1]) : 1;
      Candidate c;
      c.n_cell = nc;
      c.rows = std::max<int64_t>(1, std::min<int64_t>(row_limit, kCellTileBytes / cell_bytes));
      c.stretch = c.rows * std::min(src_row, dst_row);
      if (c.stretch > best.stretch) best = c;
    }
  }
  if (best.n_cell == 0) return false;
  if (opt.cell_form == 1) {
    // Worth it where the body that would otherwise run moves short stretches and cells make them at least twice as
    // long.  Measured on 1000 paper-shaped problems (MI355X, every qualifying step forced either way): against a
    // row-staged body that moves 16-byte vectors on both sides, cells win below 512 bytes (1.05 to 3 times; at 512
    // and more they lose 2-5 %); against its forms with narrower vectors, below 2 KiB (1.05-1.4 times); with
    // 4-byte granules, whose destination vectors are put together from four staging reads, only below
    // 640 bytes, and so against a row-staged body in destination-major order (which cells do not have); one cell dim
    // alone is the row-staged body's own case and 10 % slower here.
    const int64_t limit = gran == 4 || other.dest_major ? 640 : other.strong ? 512 : 2048;
    if (best.n_cell < 2 || other.stretch >= limit || best.stretch < 2 * other.stretch) return false;
  }
  const int nc = best.n_cell, m = r - nc;   // dims m .. r-1 form the cell, dim m-1 counts rows

  CellOp op;
  op.n_cell = nc;
  op.gran = gran;
  int64_t src_row = B, dst_row = B;
  for (int t = m; t < r; ++t) { src_row *= cs[(size_t)t]; dst_row *= cd[(size_t)t]; }
  op.src_row_bytes = (uint32_t)src_row;
  op.dst_row_bytes = (uint32_t)dst_row;

  // Parts of a cell.  Along a dim the destination tiles more coarsely there are cd/cs source parts (the last such
  // dim fastest in the part number); along a dim the source tiles more coarsely, cs/cd destination parts.
  std::vector<int64_t> n_sp((size_t)nc), n_dp((size_t)nc);
  for (int i = 0; i < nc; ++i) {
    const int64_t a = cs[(size_t)(m + i)], b = cd[(size_t)(m + i)];
    n_sp[(size_t)i] = std::max<int64_t>(1, b / a);
    n_dp[(size_t)i] = std::max<int64_t>(1, a / b);
    op.ps *= (int)n_sp[(size_t)i];
    op.pd *= (int)n_dp[(size_t)i];
  }

  std::map<std::vector<int64_t>, std::vector<int>> src_holders, dst_holders;
  for (int d = 0; d < ndev; ++d) {
    src_holders[std::vector<int64_t>(os.begin() + (size_t)d * r, os.begin() + (size_t)(d + 1) * r)].push_back(d);
    dst_holders[std::vector<int64_t>(od.begin() + (size_t)d * r, od.begin() + (size_t)(d + 1) * r)].push_back(d);
  }
  op.rep = (int)dst_holders.begin()->second.size();
  for (const auto& kv : dst_holders)
    if ((int)kv.second.size() != op.rep) return false;
  if ((int64_t)op.pd * op.rep > kCellMaxParts) return false;

  // byte strides of the dims in front of the cell on both sides (dim m-1 steps by one row)
  const int no = std::max(m, 1);     // with no dim in front of the cell, one row dim of extent 1 stands in
  std::vector<int64_t> ss((size_t)no), ds((size_t)no);
  {
    int64_t a = src_row, b = dst_row;
    for (int t = no - 1; t >= 0; --t) {
      ss[(size_t)t] = a;
      ds[(size_t)t] = b;
      if (t < m) { a *= cs[(size_t)t]; b *= cd[(size_t)t]; }
    }
  }

  // Boxes: per dim in front of the cell, the stretches between consecutive tile boundaries of either side; per cell
  // dim, the cells of the global extent.
  struct Range { int64_t lo, hi; };
  std::vector<std::vector<Range>> ranges((size_t)r);
  for (int t = 0; t < r; ++t) {
    if (t >= m) {
      const int64_t e = std::max(cs[(size_t)t], cd[(size_t)t]);
      for (int64_t lo = 0; lo < G[(size_t)t]; lo += e) ranges[(size_t)t].push_back(Range{lo, lo + e});
    } else {
      int64_t lo = 0;
      while (lo < G[(size_t)t]) {
        const int64_t hi = std::min({G[(size_t)t], (lo / cs[(size_t)t] + 1) * cs[(size_t)t], (lo / cd[(size_t)t] + 1) * cd[(size_t)t]});
        ranges[(size_t)t].push_back(Range{lo, hi});
        lo = hi;
      }
    }
  }
  std::vector<HostCellBox> hb;
  std::vector<size_t> idx((size_t)r, 0);
  while (true) {
    HostCellBox b;
    std::vector<int64_t> skey((size_t)r), dkey((size_t)r);
    for (int t = 0; t < m; ++t) {
      const Range& g = ranges[(size_t)t][idx[(size_t)t]];
      skey[(size_t)t] = g.lo / cs[(size_t)t] * cs[(size_t)t];
      dkey[(size_t)t] = g.lo / cd[(size_t)t] * cd[(size_t)t];
      b.src_off += (g.lo - skey[(size_t)t]) * ss[(size_t)t];
      b.dst_off += (g.lo - dkey[(size_t)t]) * ds[(size_t)t];
      b.len.push_back(g.hi - g.lo);
    }
    if (m == 0) b.len.push_back(1);
    b.src_first = (int32_t)op.dev_list.size();
    for (int s = 0; s < op.ps; ++s) {            // source part s: digits over n_sp, the last dim fastest
      int rest = s;
      for (int i = nc - 1; i >= 0; --i) {
        const int t = m + i;
        skey[(size_t)t] = ranges[(size_t)t][idx[(size_t)t]].lo + (rest % n_sp[(size_t)i]) * cs[(size_t)t];
        rest /= (int)n_sp[(size_t)i];
      }
      auto it = src_holders.find(skey);
      if (it == src_holders.end()) return false;
      op.dev_list.push_back(it->second.front());
    }
    b.dst_first = (int32_t)op.dev_list.size();
    for (int q = 0; q < op.pd; ++q) {
      int rest = q;
      for (int i = nc - 1; i >= 0; --i) {
        const int t = m + i;
        dkey[(size_t)t] = ranges[(size_t)t][idx[(size_t)t]].lo + (rest % n_dp[(size_t)i]) * cd[(size_t)t];
        rest /= (int)n_dp[(size_t)i];
      }
      auto it = dst_holders.find(dkey);
      if (it == dst_holders.end()) return false;
      op.dev_list.insert(op.dev_list.end(), it->second.begin(), it->second.end());
    }
    hb.push_back(std::move(b));
    int t = r - 1;
    while (t >= 0 && ++idx[(size_t)t] == ranges[(size_t)t].size()) idx[(size_t)t--] = 0;
    if (t < 0) break;
  }

  // Drop dims of extent 1 in front of the row dim; merge a dim into its predecessor when every box covers both
  // as one contiguous range on both sides.  The row dim (the last) is kept even at extent 1.
  std::vector<int64_t> kss, kds;
  std::vector<std::vector<int64_t>> klen(hb.size());
  for (int t = 0; t < no; ++t) {
    const bool row_dim = t == no - 1;
    bool all_one = true;
    for (const auto& b : hb) all_one = all_one && b.len[(size_t)t] == 1;
    if (all_one && !row_dim) continue;
    bool merged = false;
    if (!kss.empty()) {
      bool same = true;
      const int64_t l0 = hb.front().len[(size_t)t];
      for (const auto& b : hb) same = same && b.len[(size_t)t] == l0;
      if (same && kss.back() == ss[(size_t)t] * l0 && kds.back() == ds[(size_t)t] * l0) {
        for (size_t q = 0; q < hb.size(); ++q) klen[q].back() *= l0;
        kss.back() = ss[(size_t)t];
        kds.back() = ds[(size_t)t];
        merged = true;
      }
    }
    if (!merged) {
      kss.push_back(ss[(size_t)t]);
      kds.push_back(ds[(size_t)t]);
      for (size_t q = 0; q < hb.size(); ++q) klen[q].push_back(hb[q].len[(size_t)t]);
    }
  }
  op.n_outer = (int)kss.size();
  if (op.n_outer < 1 || op.n_outer > kMaxOuter) return false;
  for (int k = 0; k < kMaxOuter; ++k) { op.sstride[k] = 0; op.dstride[k] = 0; }
  for (int k = 0; k < op.n_outer; ++k) { op.sstride[k] = kss[(size_t)k]; op.dstride[k] = kds[(size_t)k]; }

  // rows per tile: what the staging area holds (parts are 16 bytes apart at least), not more than the longest box has
  int64_t cell_bytes = B;
  for (int t = m; t < r; ++t) cell_bytes *= std::max(cs[(size_t)t], cd[(size_t)t]);
  int64_t max_rows = 1;
  for (const auto& l : klen) max_rows = std::max(max_rows, l.back());
  int64_t n = std::max<int64_t>(1, std::min<int64_t>(max_rows, kCellTileBytes / cell_bytes));
  auto pitch_of = [&](int64_t rows) { return (rows * src_row + 15) / 16 * 16; };
  while (n > 1 && pitch_of(n) * op.ps > kCellTileBytes) --n;
  // tiles of a box end on 128-byte (else 64-byte) boundaries of the destination stretches where that many rows fit
  for (int64_t line : {128, 64}) {
    const int64_t al = line / std::gcd<int64_t>(dst_row, line);
    if (n / al * al * 8 >= n * 7) { n = n / al * al; break; }   // (smaller tiles cost more than boundaries inside lines)
  }
  if (pitch_of(n) * op.ps > kCellTileBytes) return false;
  op.rows_per_tile = (uint32_t)n;
  op.part_pitch = (uint32_t)pitch_of(n);

  // vector widths: what row lengths, offsets and strides allow on each side
  int vs = pow2_gcd(src_row, 16), vd = pow2_gcd(dst_row, 16);
  for (int k = 0; k < op.n_outer; ++k) { vs = pow2_gcd(op.sstride[k], vs); vd = pow2_gcd(op.dstride[k], vd); }
  for (const auto& b : hb) { vs = pow2_gcd(b.src_off, vs); vd = pow2_gcd(b.dst_off, vd); }
  // (the kernels are instantiated for side vectors of 16 bytes or one granule)
  if (vs != 16) vs = gran;
  if (vd != 16) vd = gran;
  // destination vectors narrower than 16 bytes: measured 12-22 % slower than the row-staged body
  if (opt.cell_form == 1 && vd != 16) return false;
  if (src_row % vs || dst_row % vd) return false;
  op.vs = vs;
  op.vd = vd;
  uint8_t sh = 0;
  op.spv = (uint32_t)(n * src_row / vs);
  magic_for(op.spv, &op.spv_magic, &sh); op.spv_shift = sh;
  op.dpv = (uint32_t)(n * dst_row / vd);
  magic_for(op.dpv, &op.dpv_magic, &sh); op.dpv_shift = sh;
  op.drow_gran = (uint32_t)(dst_row / gran);
  magic_for(op.drow_gran, &op.drg_magic, &sh); op.drg_shift = sh;

  // Staging addresses.  Entry i of the per-dim arrays is cell dim r-1-i (the last dim first, counted in granules).
  for (int i = 0; i < kMaxCellDims; ++i) {
    op.dext[i] = 1; op.dext_magic[i] = 0; op.dext_shift[i] = 0;
    op.piece[i] = 0; op.piece_magic[i] = 0; op.piece_shift[i] = 0;
    op.lds_step[i] = 0; op.part_step[i] = 0;
  }
  {
    int64_t step = gran, part_weight = 1;
    for (int i = 0; i < nc; ++i) {
      const int t = r - 1 - i;
      const int64_t unit = i == 0 ? B : 1, per = i == 0 ? gran : 1;   // the last dim counts granules
      const int64_t a = cs[(size_t)t] * unit / per, b = cd[(size_t)t] * unit / per;
      op.dext[i] = (uint32_t)b;
      magic_for(op.dext[i], &op.dext_magic[i], &sh); op.dext_shift[i] = sh;
      op.lds_step[i] = (uint32_t)step;
      if (b > a) {
        op.piece[i] = (uint32_t)a;
        magic_for(op.piece[i], &op.piece_magic[i], &sh); op.piece_shift[i] = sh;
        op.part_step[i] = (uint32_t)(part_weight * op.part_pitch);
        part_weight *= b / a;
      }
      step *= a;
    }
  }
  // first granule of destination part q in the staging area: along a dim the source tiles more coarsely, part
  // digit times the destination tile's extent
  op.base_first = (int32_t)op.dev_list.size();
  for (int q = 0; q < op.pd; ++q) {
    int rest = q;
    int64_t base = 0;
    for (int i = 0; i < nc; ++i) {             // the last dim is the fastest digit of q
      const int ci = nc - 1 - i;               // index into n_dp (dim order)
      const int64_t digit = rest % n_dp[(size_t)ci];
      rest /= (int)n_dp[(size_t)ci];
      base += digit * op.dext[i] * op.lds_step[i];
    }
    op.dev_list.push_back((int32_t)base);
  }

  op.max_grid = std::max(1u, std::min(opt.max_grid, 16777215u));
  uint64_t tiles = 0;
  bool uniform = true;
  int64_t min_rows = INT64_MAX;
  for (size_t q = 0; q < hb.size(); ++q) {
    DevCellBox db{};
    db.src_off = hb[q].src_off;
    db.dst_off = hb[q].dst_off;
    db.src_first = hb[q].src_first;
    db.dst_first = hb[q].dst_first;
    int64_t rows_total = 1, outer = 1;
    for (int k = 0; k < op.n_outer; ++k) {
      const int64_t l = klen[q][(size_t)k];
      if (l >= (1ll << 31)) return false;
      db.len[k] = (uint32_t)l;
      magic_for((uint32_t)l, &db.magic[k], &db.shift[k]);
      rows_total *= l;
      if (k + 1 < op.n_outer) outer *= l;
    }
    const int64_t row_len = klen[q].back(), row_tiles = (row_len + n - 1) / n;
    min_rows = std::min(min_rows, std::min(row_len, n));
    if (outer * row_tiles >= (1ll << 31)) return false;
    db.row_tiles = (uint32_t)row_tiles;
    magic_for(db.row_tiles, &db.rt_magic, &db.rt_shift);
    db.n_tiles = (uint32_t)(outer * row_tiles);
    db.tile_first = (uint32_t)tiles;
    tiles += db.n_tiles;
    if (tiles >= (1ull << 31)) return false;
    if (!op.boxes.empty() && db.n_tiles != op.boxes.front().n_tiles) uniform = false;
    op.boxes.push_back(db);
    op.bytes_read += rows_total * src_row * op.ps;
    op.bytes_written += rows_total * dst_row * op.pd * op.rep;
  }
  op.n_tiles = (uint32_t)tiles;
  op.tiles_per_box = (uniform && !op.boxes.empty()) ? op.boxes.front().n_tiles : 0;
  if (op.tiles_per_box > 1) {
    magic_for(op.tiles_per_box, &op.tpb_magic, &sh);
    op.tpb_shift = sh;
  }
  op.min_stretch = min_rows * std::min(src_row, dst_row);
  if (opt.cell_form == 1 && op.min_stretch < 2 * other.stretch) return false;
  op.enabled = true;
  *out = std::move(op);
  return true;
}

}  // namespace redist
