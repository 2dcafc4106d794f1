// Planner for type-directed array redistribution (arXiv 2112.01075).
//
//   1. validate the problem                       (Fig. "Well-formedness rules", Sec. 2.5)
//   2. decompose every mesh axis into prime axes  (Sec. 3, Principle 1)
//   3. shortest path over weak types              (Sec. 7.2; weights: Fig. cost model;
//      nodes = local types within the memory bound of Eq. (3); label strings restricted to
//      the normal form dynslice* alltoall* allgather* of Def. 4.5, which loses no cost by the
//      lemma on normal forms of weak sequences)
//   4. lowering to device-level collectives       (Sec. 6.1): the state is the table
//      "physical device -> base offset of the tile it holds" (beta o phi^-1, the only physically
//      meaningful part of a device assignment).  allgather / alltoall act on the groups of
//      devices holding the adjacent tiles of an aligned super-tile, so their effect on the table
//      is a function of the table; the only freedom is which unused axes a dynslice takes.
//   5. the axes for dynslices are picked with a bias towards the target type and verified by
//      simulating the offset tables; a final allpermute is added only if the reached table
//      differs from T[[dst]], and it is hoisted in front of the trailing allgathers (Sec. 7.3).
#include "planner.hpp"

#include <algorithm>
#include <functional>
#include <map>
#include <queue>
#include <set>
#include <tuple>

namespace redist {

int64_t product(const std::vector<int64_t>& v) {
  int64_t p = 1;
  for (int64_t x : v) p *= x;
  return p;
}

namespace {

using Shape = std::vector<int64_t>;
using PrimeBag = std::map<int64_t, int>;  // prime -> multiplicity

std::vector<int64_t> factorize(int64_t n) {
  std::vector<int64_t> f;
  for (int64_t p = 2; p * p <= n; ++p)
    while (n % p == 0) { f.push_back(p); n /= p; }
  if (n > 1) f.push_back(n);
  return f;
}

PrimeBag bag_of(int64_t n) {
  PrimeBag b;
  for (int64_t p : factorize(n)) b[p]++;
  return b;
}

// All products (> 1) of sub-multisets of a prime bag.
std::vector<int64_t> divisors_of_bag(const PrimeBag& bag) {
  std::vector<int64_t> out{1};
  for (const auto& pm : bag) {
    size_t n = out.size();
    int64_t pw = 1;
    for (int e = 1; e <= pm.second; ++e) {
      pw *= pm.first;
      for (size_t k = 0; k < n; ++k) out.push_back(out[k] * pw);
    }
  }
  out.erase(std::remove(out.begin(), out.end(), (int64_t)1), out.end());
  std::sort(out.begin(), out.end());
  return out;
}

// The mesh after prime decomposition.  Prime axis p of original axis a carries the digit of
// weight prod(previous primes of a) in a's coordinate, so shard indices are unchanged.
struct PrimeMesh {
  std::vector<int64_t> size;    // prime size of each prime axis
  std::vector<int64_t> stride;  // shard-index stride of its coordinate
  int ndev = 1;
  int coord(int dev, int ax) const { return (int)((dev / stride[ax]) % size[ax]); }
};

using AxisLists = std::vector<std::vector<int>>;  // per dim: prime axis ids, minor-to-major

struct State {
  Shape shape;                // local tile shape
  std::vector<int64_t> offs;  // ndev*rank
};

// T[[type]] for every physical device under the identity device map (Fig. "Base offset maps").
std::vector<int64_t> offsets_of(const PrimeMesh& pm, const AxisLists& lists, const Shape& shape) {
  int r = (int)shape.size();
  std::vector<int64_t> offs((size_t)pm.ndev * r, 0);
  for (int d = 0; d < pm.ndev; ++d)
    for (int t = 0; t < r; ++t) {
      int64_t w = shape[t], o = 0;
      for (int ax : lists[t]) { o += w * pm.coord(d, ax); w *= pm.size[ax]; }
      offs[(size_t)d * r + t] = o;
    }
  return offs;
}

struct WeakStep { int kind, i, j; int64_t f; };

bool operator<(const WeakStep& a, const WeakStep& b) {
  return std::tie(a.kind, a.i, a.j, a.f) < std::tie(b.kind, b.i, b.j, b.f);
}

int phase_of(int kind) { return kind == kDynSlice ? 0 : (kind == kAllToAll ? 1 : 2); }

// ---- device-table effect of each collective ------------------------------------------------
// dynslice(i, f) with the unused prime axes xs (first = minor-most): device keeps chunk
// m = mixed-radix value of its coordinates on xs.
void apply_dynslice(const PrimeMesh& pm, State* s, int i, int64_t f, const std::vector<int>& xs) {
  int r = (int)s->shape.size();
  int64_t c = s->shape[i] / f;
  for (int d = 0; d < pm.ndev; ++d) {
    int64_t m = 0, w = 1;
    for (int ax : xs) { m += w * pm.coord(d, ax); w *= pm.size[ax]; }
    s->offs[(size_t)d * r + i] += m * c;
  }
  s->shape[i] = c;
}

// allgather(i, f): the f holders of the adjacent tiles of an aligned super-tile all end with it.
void apply_allgather(State* s, int i, int64_t f) {
  int r = (int)s->shape.size();
  int64_t big = s->shape[i] * f;
  for (size_t d = 0; d * r < s->offs.size(); ++d) {
    int64_t& o = s->offs[d * r + i];
    o = (o / big) * big;
  }
  s->shape[i] = big;
}

// alltoall(i -> j, f): the holder of sub-tile p (along i) of a super-tile ends with chunk p
// (along j) of the super-tile.
void apply_alltoall(State* s, int i, int j, int64_t f) {
  int r = (int)s->shape.size();
  int64_t ci = s->shape[i], cj = s->shape[j] / f;
  for (size_t d = 0; d * r < s->offs.size(); ++d) {
    int64_t& oi = s->offs[d * r + i];
    int64_t p = (oi / ci) % f;
    oi -= p * ci;
    s->offs[d * r + j] += p * cj;
  }
  s->shape[i] = ci * f;
  s->shape[j] = cj;
}

// ---- weak shortest-path search ---------------------------------------------------------------
struct SearchNode {
  Shape c;
  int phase;
  int64_t dist;
  std::vector<std::pair<int, WeakStep>> preds;  // tight incoming edges (predecessor node id, step)
};

class WeakSearch {
 public:
  // latency: elements added to the weight of every step that communicates (0 = the paper's cost model)
  WeakSearch(const Shape& gshape, const PrimeBag& mesh_bag, const Shape& c1, const Shape& c2, int64_t latency)
      : g_(gshape), mesh_(mesh_bag), c1_(c1), c2_(c2), r_((int)gshape.size()), lat_(latency) {
    bound_ = std::max(product(c1), product(c2));
  }

  // Returns up to max_paths optimal normal-form step lists, fewest steps first.
  uint32_t limits_hit = 0;   // bit 0: more optimal paths than max_paths; bit 1: visit limit of the enumeration

  bool run(std::vector<std::vector<WeakStep>>* paths, int64_t* best_cost, size_t max_paths) {
    const int64_t INF = INT64_MAX;
    int start = node_id(c1_, 0);
    nodes_[start].dist = 0;
    using QE = std::tuple<int64_t, int>;
    std::priority_queue<QE, std::vector<QE>, std::greater<QE>> pq;
    pq.push({0, start});
    int64_t best = INF;
    while (!pq.empty()) {
      const int64_t du = std::get<0>(pq.top());
      const int u = std::get<1>(pq.top());
      pq.pop();
      if (du > nodes_[u].dist) continue;
      if (du > best) break;
      if (nodes_[u].c == c2_) best = std::min(best, du);
      Shape cu = nodes_[u].c;  // copy: nodes_ may reallocate below
      int pu = nodes_[u].phase;
      for_each_edge(cu, pu, [&](const WeakStep& st, const Shape& nc, int64_t w) {
        int v = node_id(nc, phase_of(st.kind));
        int64_t nd = du + w;
        if (nd < nodes_[v].dist) {
          nodes_[v].dist = nd;
          nodes_[v].preds.clear();
          nodes_[v].preds.push_back({u, st});
          pq.push({nd, v});
        } else if (nd == nodes_[v].dist) {
          nodes_[v].preds.push_back({u, st});
        }
      });
    }
    if (best == INF) return false;
    *best_cost = best;
    // enumerate tight paths backwards from every goal node of optimal cost
    std::vector<WeakStep> suffix;
    size_t visits = 0;
    std::function<void(int)> dfs = [&](int v) {
      if (paths->size() >= max_paths) { limits_hit |= 1u; return; }
      if (++visits > 200000) { limits_hit |= 2u; return; }
      if (v == start) {
        paths->push_back(std::vector<WeakStep>(suffix.rbegin(), suffix.rend()));
        return;
      }
      if (suffix.size() >= 24) return;
      auto preds = nodes_[v].preds;
      std::sort(preds.begin(), preds.end(), [](const auto& a, const auto& b) { return a.second < b.second; });
      for (const auto& pe : preds) {
        const WeakStep& e = pe.second;
        if (!suffix.empty()) {
          const WeakStep& nx = suffix.back();  // the step that follows e
          // zero-cost slices on different dims commute and merge per dim: keep one canonical order
          // (gathers do not: gathering the smaller factor first is cheaper)
          if (e.kind == kDynSlice && nx.kind == kDynSlice && e.i >= nx.i) continue;
        }
        suffix.push_back(e);
        dfs(pe.first);
        suffix.pop_back();
      }
    };
    for (int ph = 0; ph < 3; ++ph) {
      auto it = index_.find({c2_, ph});
      if (it != index_.end() && nodes_[it->second].dist == best) dfs(it->second);
    }
    std::stable_sort(paths->begin(), paths->end(),
                     [](const auto& a, const auto& b) { return a.size() < b.size(); });
    return !paths->empty();
  }

 private:
  int node_id(const Shape& c, int phase) {
    auto key = std::make_pair(c, phase);
    auto it = index_.find(key);
    if (it != index_.end()) return it->second;
    int id = (int)nodes_.size();
    nodes_.push_back(SearchNode{c, phase, INT64_MAX, {}});
    index_[key] = id;
    return id;
  }

  template <class F>
  void for_each_edge(const Shape& c, int phase, F&& emit) {
    int64_t L = product(c);
    PrimeBag free = mesh_;
    for (int t = 0; t < r_; ++t)
      for (int64_t p : factorize(g_[t] / c[t])) free[p]--;
    for (auto it = free.begin(); it != free.end();) it = (it->second <= 0) ? free.erase(it) : std::next(it);
    std::vector<int64_t> free_div = divisors_of_bag(free);
    for (int i = 0; i < r_; ++i) {
      if (phase == 0)
        for (int64_t f : free_div)
          if (c[i] % f == 0) {
            Shape n = c;
            n[i] /= f;
            emit(WeakStep{kDynSlice, i, -1, f}, n, (int64_t)0);
          }
      for (int64_t f : divisors_of_bag(bag_of(g_[i] / c[i]))) {
        if (L * f <= bound_) {
          Shape n = c;
          n[i] *= f;
          emit(WeakStep{kAllGather, i, -1, f}, n, L * f + lat_);
        }
        if (phase <= 1)
          for (int j = 0; j < r_; ++j)
            if (j != i && c[j] % f == 0) {
              Shape n = c;
              n[i] *= f;
              n[j] /= f;
              emit(WeakStep{kAllToAll, i, j, f}, n, L + lat_);
            }
      }
    }
  }

  Shape g_;
  PrimeBag mesh_;
  Shape c1_, c2_;
  int r_;
  int64_t lat_;
  int64_t bound_;
  std::vector<SearchNode> nodes_;
  std::map<std::pair<Shape, int>, int> index_;
};

// ---- choosing the axes of the dynslices (Sec. 7.3, second optimisation) -------------------------
// All ordered tuples of distinct axes from `pool` whose sizes multiply to f.
void axis_tuples(const PrimeMesh& pm, const std::vector<int>& pool, int64_t f, std::vector<int>* cur,
                 std::vector<std::vector<int>>* out) {
  if (f == 1) {
    if (!cur->empty()) out->push_back(*cur);
    return;
  }
  if (out->size() > 5000) return;
  for (int ax : pool) {
    if (f % pm.size[ax]) continue;
    if (std::find(cur->begin(), cur->end(), ax) != cur->end()) continue;
    cur->push_back(ax);
    axis_tuples(pm, pool, f / pm.size[ax], cur, out);
    cur->pop_back();
  }
}

// Preference of prepending xs to dim i (current list `have`), given the target list `want`:
// how long a suffix of want the new list xs++have reproduces, then how many of xs the target uses
// on this dim, then how many it leaves unused anywhere.
std::tuple<int, int, int> tuple_score(const std::vector<int>& xs, const std::vector<int>& have,
                                      const std::vector<int>& want, const std::set<int>& dst_used) {
  std::vector<int> now = xs;
  now.insert(now.end(), have.begin(), have.end());
  int suffix = 0;
  while (suffix < (int)now.size() && suffix < (int)want.size() &&
         now[now.size() - 1 - suffix] == want[want.size() - 1 - suffix])
    ++suffix;
  int on_dim = 0, unused = 0;
  for (int ax : xs) {
    if (std::find(want.begin(), want.end(), ax) != want.end()) ++on_dim;
    if (!dst_used.count(ax)) ++unused;
  }
  return {suffix, on_dim, unused};
}

struct Lowering {
  std::vector<WeakStep> path;
  std::vector<std::vector<int>> slice_axes;  // per dynslice step of path, the axes taken
  std::vector<State> states;                 // after each step
  bool exact = false;                        // final table == T[[dst]]
};

void simulate(const PrimeMesh& pm, const State& start, Lowering* lo) {
  lo->states.clear();
  State s = start;
  size_t si = 0;
  for (const WeakStep& st : lo->path) {
    if (st.kind == kDynSlice) apply_dynslice(pm, &s, st.i, st.f, lo->slice_axes[si++]);
    else if (st.kind == kAllGather) apply_allgather(&s, st.i, st.f);
    else apply_alltoall(&s, st.i, st.j, st.f);
    lo->states.push_back(s);
  }
}

// ---- groups / peers ----------------------------------------------------------------------------
// For allgather/alltoall(i, f) on table `s`: devices holding the same sub-tile are replicas; the
// r-th replica of every sub-tile of a super-tile forms one group.  peers[d*f + rank] = member.
bool group_peers(const State& s, int ndev, int i, int64_t f, std::vector<int32_t>* peers) {
  int r = (int)s.shape.size();
  int64_t ci = s.shape[i], big = ci * f;
  std::map<std::vector<int64_t>, std::vector<std::vector<int>>> by_super;  // key -> per sub-pos holders
  for (int d = 0; d < ndev; ++d) {
    std::vector<int64_t> key(s.offs.begin() + (size_t)d * r, s.offs.begin() + (size_t)(d + 1) * r);
    int64_t p = (key[i] / ci) % f;
    key[i] = (key[i] / big) * big;
    auto& slots = by_super[key];
    if (slots.empty()) slots.resize((size_t)f);
    slots[(size_t)p].push_back(d);
  }
  peers->assign((size_t)ndev * f, -1);
  for (auto& kv : by_super) {
    auto& slots = kv.second;
    size_t reps = slots[0].size();
    for (auto& h : slots)
      if (h.size() != reps || reps == 0) return false;
    for (size_t g = 0; g < reps; ++g)
      for (int64_t p = 0; p < f; ++p) {
        int member = slots[(size_t)p][g];
        for (int64_t q = 0; q < f; ++q) (*peers)[(size_t)member * f + q] = slots[(size_t)q][g];
      }
  }
  return true;
}

std::vector<int64_t> row(const std::vector<int64_t>& offs, int d, int r) {
  return std::vector<int64_t>(offs.begin() + (size_t)d * r, offs.begin() + (size_t)(d + 1) * r);
}

// Bijection src[d] such that device d receives a tile with base offset want[d] from the table
// have (both balanced covers with the same tile shape).  Devices already holding what they need
// keep it; the rest are matched in device order.
bool match_permutation(const std::vector<int64_t>& have, const std::vector<int64_t>& want, int ndev, int r,
                       std::vector<int32_t>* src) {
  std::map<std::vector<int64_t>, std::vector<int>> holders;
  src->assign((size_t)ndev, -1);
  std::vector<char> taken((size_t)ndev, 0);
  for (int d = 0; d < ndev; ++d)
    if (row(have, d, r) == row(want, d, r)) { (*src)[d] = d; taken[d] = 1; }
  for (int d = ndev - 1; d >= 0; --d)
    if (!taken[d]) holders[row(have, d, r)].push_back(d);  // pop_back yields ascending order
  for (int d = 0; d < ndev; ++d) {
    if ((*src)[d] >= 0) continue;
    auto it = holders.find(row(want, d, r));
    if (it == holders.end() || it->second.empty()) return false;
    (*src)[d] = it->second.back();
    it->second.pop_back();
  }
  return true;
}

Status validate_type(const std::vector<int64_t>& mesh, const TypeSpec& t, std::vector<char>* used) {
  int r = (int)t.gshape.size();
  if (r < 1 || r > kMaxRank || (int)t.axes.size() != r) return kErrIllFormed;
  for (int k = 0; k < r; ++k) {
    if (t.gshape[k] < 1) return kErrIllFormed;
    int64_t tiles = 1;
    for (int ax : t.axes[k]) {
      if (ax < 0 || ax >= (int)mesh.size()) return kErrIllFormed;   // axis not in the mesh
      if ((*used)[ax]) return kErrIllFormed;                        // axis used twice (affine use)
      (*used)[ax] = 1;
      tiles *= mesh[ax];
    }
    if (t.gshape[k] % tiles) return kErrIllFormed;                  // c * prod(k) = n has no solution
  }
  return kOk;
}

}  // namespace

Status make_plan(const std::vector<int64_t>& mesh, const TypeSpec& src, const TypeSpec& dst, int elem_size,
                 int mode, int64_t step_latency_elems, PlanCore* out) {
  if (mesh.empty()) return kErrBadMesh;
  int64_t ndev64 = 1;
  for (int64_t k : mesh) {
    if (k < 1) return kErrBadMesh;
    ndev64 *= k;
    if (ndev64 > kMaxDevices) return kErrBadMesh;
  }
  if (elem_size != 1 && elem_size != 2 && elem_size != 4 && elem_size != 8 && elem_size != 16)
    return kErrBadElemSize;
  if (mode != kStepwise && mode != kFusedMode && mode != kNaive) return kErrBadArg;
  {
    std::vector<char> u1(mesh.size(), 0), u2(mesh.size(), 0);
    if (Status s = validate_type(mesh, src, &u1)) return s;
    if (Status s = validate_type(mesh, dst, &u2)) return s;
  }
  if (src.gshape != dst.gshape) return kErrGlobalMismatch;

  const int ndev = (int)ndev64, r = (int)src.gshape.size();

  // prime decomposition: axis a -> primes ascending, minor to major
  PrimeMesh pm;
  pm.ndev = ndev;
  std::vector<std::vector<int>> primes_of(mesh.size());
  PrimeBag mesh_bag;
  {
    int64_t stride = 1;
    for (int a = (int)mesh.size() - 1; a >= 0; --a) {
      int64_t w = stride;
      for (int64_t p : factorize(mesh[a])) {
        primes_of[a].push_back((int)pm.size.size());
        pm.size.push_back(p);
        pm.stride.push_back(w);
        w *= p;
        mesh_bag[p]++;
      }
      stride *= mesh[a];
    }
  }
  auto lists_of = [&](const TypeSpec& t) {
    AxisLists l(r);
    for (int k = 0; k < r; ++k)
      for (int a : t.axes[k])
        for (int p : primes_of[a]) l[k].push_back(p);
    return l;
  };
  auto shape_of = [&](const AxisLists& l) {
    Shape c(r);
    for (int k = 0; k < r; ++k) {
      int64_t tiles = 1;
      for (int ax : l[k]) tiles *= pm.size[ax];
      c[k] = src.gshape[k] / tiles;
    }
    return c;
  };
  AxisLists l1 = lists_of(src), l2 = lists_of(dst);
  Shape c1 = shape_of(l1), c2 = shape_of(l2);

  PlanCore pc;
  pc.ndev = ndev; pc.rank = r; pc.elem_size = elem_size; pc.mode = mode;
  pc.gshape = src.gshape;
  pc.shape_src = c1; pc.shape_dst = c2;
  pc.offs_src = offsets_of(pm, l1, c1);
  pc.offs_dst = offsets_of(pm, l2, c2);
  pc.bound = std::max(product(c1), product(c2));
  const State start{c1, pc.offs_src};

  auto push_step = [&](int kind, int i, int j, int64_t f, const State& after) -> Step& {
    Step st;
    st.kind = kind; st.dim_i = i; st.dim_j = j; st.factor = f;
    st.shape_after = after.shape;
    st.offs_after = after.offs;
    pc.steps.push_back(std::move(st));
    return pc.steps.back();
  };

  if (mode == kFusedMode) {
    push_step(kFused, -1, -1, 1, State{c2, pc.offs_dst});
  } else if (mode == kNaive) {
    // Eq. (2): gather every tiled dim of src completely, then slice every tiled dim of dst.
    State s = start;
    for (int k = 0; k < r; ++k)
      if (!l1[k].empty()) {
        int64_t f = src.gshape[k] / s.shape[k];
        std::vector<int32_t> peers;
        if (!group_peers(s, ndev, k, f, &peers)) return kErrInternal;
        apply_allgather(&s, k, f);
        push_step(kAllGather, k, -1, f, s).peers = std::move(peers);
      }
    for (int k = 0; k < r; ++k)
      if (!l2[k].empty()) {
        int64_t f = s.shape[k] / c2[k];
        State before = s;
        apply_dynslice(pm, &s, k, f, l2[k]);
        Step& st = push_step(kDynSlice, k, -1, f, s);
        st.peers.resize(ndev);
        for (int d = 0; d < ndev; ++d)
          st.peers[d] = (int32_t)((s.offs[(size_t)d * r + k] - before.offs[(size_t)d * r + k]) / s.shape[k]);
      }
    if (s.offs != pc.offs_dst || s.shape != c2) return kErrInternal;
  } else {
    // ---- weak shortest paths ----
    std::vector<std::vector<WeakStep>> paths;
    int64_t weak_cost = 0;
    if (c1 == c2) {
      paths.push_back({});
    } else {
      WeakSearch ws(src.gshape, mesh_bag, c1, c2, step_latency_elems);
      if (!ws.run(&paths, &weak_cost, 64)) return kErrSearchBudget;
      pc.limits_hit |= ws.limits_hit;
    }
    // ---- lowering: pick dynslice axes, prefer a lowering that needs no allpermute ----
    std::set<int> src_used, dst_used;
    for (auto& l : l1) src_used.insert(l.begin(), l.end());
    for (auto& l : l2) dst_used.insert(l.begin(), l.end());
    Lowering chosen;
    bool have_choice = false;
    int budget = 4096;
    for (const auto& path : paths) {
      if (budget <= 0 || (have_choice && chosen.exact)) break;
      std::vector<int> slice_idx;
      for (size_t k = 0; k < path.size(); ++k)
        if (path[k].kind == kDynSlice) slice_idx.push_back((int)k);
      Lowering lo;
      lo.path = path;
      lo.slice_axes.assign(slice_idx.size(), {});
      std::function<bool(size_t, std::set<int>, AxisLists)> rec = [&](size_t n, std::set<int> used,
                                                                      AxisLists lists) -> bool {
        if (budget <= 0) return false;
        if (n == slice_idx.size()) {
          --budget;
          simulate(pm, start, &lo);
          const State& fin = lo.states.empty() ? start : lo.states.back();
          lo.exact = (fin.offs == pc.offs_dst);
          if (!have_choice || lo.exact) { chosen = lo; have_choice = true; }
          return lo.exact;
        }
        const WeakStep& st = path[(size_t)slice_idx[n]];
        std::vector<int> pool;
        for (int ax = 0; ax < (int)pm.size.size(); ++ax)
          if (!used.count(ax)) pool.push_back(ax);
        std::vector<std::vector<int>> cands;
        std::vector<int> cur;
        axis_tuples(pm, pool, st.f, &cur, &cands);
        std::stable_sort(cands.begin(), cands.end(), [&](const auto& a, const auto& b) {
          return tuple_score(a, lists[st.i], l2[st.i], dst_used) > tuple_score(b, lists[st.i], l2[st.i], dst_used);
        });
        for (const auto& xs : cands) {
          std::set<int> u2 = used;
          u2.insert(xs.begin(), xs.end());
          AxisLists nl = lists;
          nl[st.i].insert(nl[st.i].begin(), xs.begin(), xs.end());
          lo.slice_axes[n] = xs;
          if (rec(n + 1, u2, nl)) return true;
        }
        return false;
      };
      rec(0, src_used, l1);
    }
    if (!have_choice) return kErrInternal;
    if (budget <= 0 && !chosen.exact) pc.limits_hit |= 4u;

    // ---- emit steps; add the single allpermute if needed, in front of the trailing allgathers ----
    size_t n_steps = chosen.path.size();
    size_t first_gather = n_steps;
    while (first_gather > 0 && chosen.path[first_gather - 1].kind == kAllGather) --first_gather;
    State s = start;
    size_t si = 0;
    auto emit_weak = [&](const WeakStep& w) -> Status {
      if (w.kind == kDynSlice) {
        State before = s;
        apply_dynslice(pm, &s, w.i, w.f, chosen.slice_axes[si++]);
        Step& st = push_step(kDynSlice, w.i, -1, w.f, s);
        st.peers.resize(ndev);
        for (int d = 0; d < ndev; ++d)
          st.peers[d] = (int32_t)((s.offs[(size_t)d * r + w.i] - before.offs[(size_t)d * r + w.i]) / s.shape[w.i]);
      } else {
        std::vector<int32_t> peers;
        if (!group_peers(s, ndev, w.i, w.f, &peers)) return kErrInternal;
        if (w.kind == kAllGather) apply_allgather(&s, w.i, w.f);
        else apply_alltoall(&s, w.i, w.j, w.f);
        push_step(w.kind, w.i, w.j, w.f, s).peers = std::move(peers);
      }
      return kOk;
    };
    for (size_t k = 0; k < first_gather; ++k)
      if (Status e = emit_weak(chosen.path[k])) return e;
    if (!chosen.exact) {
      // Table wanted in front of the gathers: device d must hold a sub-tile of its target tile,
      // every sub-tile of a target tile held equally often among that tile's devices.
      std::vector<int64_t> want((size_t)ndev * r);
      std::map<std::vector<int64_t>, std::vector<int>> by_target;
      for (int d = 0; d < ndev; ++d) by_target[row(pc.offs_dst, d, r)].push_back(d);
      for (auto& kv : by_target) {
        const std::vector<int64_t>& base = kv.first;
        std::vector<int64_t> nsub(r);
        int64_t total = 1;
        for (int t = 0; t < r; ++t) { nsub[t] = c2[t] / s.shape[t]; total *= nsub[t]; }
        int64_t cap = (int64_t)kv.second.size() / total;
        if (cap * total != (int64_t)kv.second.size()) return kErrInternal;
        std::map<std::vector<int64_t>, int64_t> left;
        std::vector<std::vector<int64_t>> subs;
        for (int64_t n = 0; n < total; ++n) {
          std::vector<int64_t> o = base;
          int64_t rem = n;
          for (int t = r - 1; t >= 0; --t) { o[t] += (rem % nsub[t]) * s.shape[t]; rem /= nsub[t]; }
          left[o] = cap;
          subs.push_back(o);
        }
        std::vector<int> pending;
        for (int d : kv.second) {
          auto it = left.find(row(s.offs, d, r));
          if (it != left.end() && it->second > 0) {
            --it->second;
            std::copy(it->first.begin(), it->first.end(), want.begin() + (size_t)d * r);
          } else {
            pending.push_back(d);
          }
        }
        size_t cursor = 0;
        for (int d : pending) {
          while (cursor < subs.size() && left[subs[cursor]] == 0) ++cursor;
          if (cursor == subs.size()) return kErrInternal;
          --left[subs[cursor]];
          std::copy(subs[cursor].begin(), subs[cursor].end(), want.begin() + (size_t)d * r);
        }
      }
      std::vector<int32_t> perm;
      if (!match_permutation(s.offs, want, ndev, r, &perm)) return kErrInternal;
      s.offs = want;
      push_step(kAllPermute, -1, -1, 1, s).peers = std::move(perm);
    }
    for (size_t k = first_gather; k < n_steps; ++k)
      if (Status e = emit_weak(chosen.path[k])) return e;
    if (s.shape != c2 || s.offs != pc.offs_dst) return kErrInternal;
  }

  // ---- accounting: Fig. cost model, Def. 4.4 ----
  int64_t L = product(c1);
  pc.height = L;
  pc.cost = pc.weak_cost = 0;
  for (const Step& st : pc.steps) {
    int64_t Ln = product(st.shape_after);
    int64_t w = 0;
    if (st.kind == kAllPermute || st.kind == kAllToAll) w = L;
    else if (st.kind == kAllGather) w = Ln;
    pc.cost += w;
    if (st.kind != kAllPermute) pc.weak_cost += w;
    pc.height = std::max(pc.height, Ln);
    L = Ln;
  }
  *out = std::move(pc);
  return kOk;
}

}  // namespace redist
