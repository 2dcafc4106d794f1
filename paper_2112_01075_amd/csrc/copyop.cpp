#include "copyop.hpp"

#include <algorithm>
#include <cstdlib>
#include <map>
#include <numeric>

namespace redist {
namespace {

struct Seg {  // one piece of a destination tile's extent in a dim, lying in one source tile
  int64_t dst_start, len, src_start, src_tile;
};

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

bool build_copy_op(int kind, int ndev, int rank, int elem_size, const std::vector<int64_t>& cs,
                   const std::vector<int64_t>& os, const std::vector<int64_t>& cd, const std::vector<int64_t>& od,
                   CopyOp* out) {
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

  struct HostBox { int64_t soff, doff; int src_dev, dst_first, dst_count; std::vector<int64_t> len; };
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
      hb.push_back(std::move(b));
      int g = ng - 1;
      while (g >= 0 && ++idx[g] == segs[g].size()) idx[g--] = 0;
      if (g < 0) break;
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
  op.vec_bytes = v;

  // ---- tiling: 256 threads x unroll vectors; as wide as the longest run allows ----
  int64_t total_vecs = 0;
  for (const auto& b : hb) {
    int64_t n = b.len[ng - 1] * elem_size / v;
    for (int k = 0; k < op.n_outer; ++k) n *= b.len[keep[k]];
    total_vecs += n;
  }
  op.unroll = 4;
  if (const char* e = std::getenv("REDIST_DEBUG_UNROLL")) {
    int u = std::atoi(e);
    if (u == 1 || u == 2 || u == 4 || u == 8) op.unroll = u;
  }
  if (const char* e = std::getenv("REDIST_DEBUG_NT")) op.nontemporal = std::atoi(e) != 0;
  if (const char* e = std::getenv("REDIST_DEBUG_LDS_KB")) op.lds_bytes = std::min(64, std::max(0, std::atoi(e))) * 1024;
  const int64_t tile_vecs = 256 * op.unroll;
  int64_t max_run_vecs = max_run_bytes / v;
  op.tc_log2 = 0;
  while ((1ll << op.tc_log2) < max_run_vecs && (1ll << op.tc_log2) < tile_vecs) ++op.tc_log2;
  const int64_t tc = 1ll << op.tc_log2, tr = tile_vecs >> op.tc_log2;

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
  op.n_tiles = (uint32_t)tiles;
  op.tiles_per_box = (uniform && !op.boxes.empty()) ? op.boxes.front().n_tiles : 0;
  if (op.tiles_per_box > 1) {
    uint8_t sh = 0;
    magic_for(op.tiles_per_box, &op.tpb_magic, &sh);
    op.tpb_shift = sh;
  }
  *out = std::move(op);
  return true;
}

}  // namespace redist
