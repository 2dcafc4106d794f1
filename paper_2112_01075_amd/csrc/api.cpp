// C-ABI of the library: argument checking, plan objects, workspace layout, kernel enqueueing.
#include <hip/hip_runtime_api.h>

#include <atomic>
#include <cstring>
#include <deque>
#include <map>
#include <mutex>
#include <memory>
#include <new>
#include <vector>

#include "../../include/redist.h"
#include "copyop.hpp"
#include "launch.hpp"
#include "planner.hpp"

using namespace redist;

struct redist_plan {
  std::atomic<int> refs{1};            // redist_plan_destroy frees at zero (the plan cache holds one reference of its own)
  BuildOptions opt;                    // how the plan was lowered to launches
  int64_t launch_latency_ns = 3000, sustained_gbs = 5500;   // the time model of REDIST_MODE_AUTO
  PlanCore core;
  std::vector<CopyOp> ops;             // one per executed kernel (>= 1 even for an empty step list)
  std::vector<int> op_last_step;       // the last plan step each launch carries out (a launch may cover a run of steps)
  std::vector<int64_t> shard_stride;   // bytes between consecutive shards of intermediate k (after op k)
  std::vector<int64_t> region_off;     // byte offset of intermediate k in the workspace
  int64_t workspace_bytes = 0;
  // Host image of the descriptors, laid out at creation: what redist_plan_prepare copies to device memory and what
  // redist_execute_static uploads to the static scratch area; offsets are relative to its start.
  std::vector<char> blob;
  std::vector<size_t> boxes_off, list_off;      // generic descriptors per op
  std::vector<size_t> rbox_off, rpiece_off, rlist_off;  // row-complete descriptors per op
  std::vector<size_t> cbox_off, clist_off;              // cell-complete descriptors per op
  // meshes beyond kMaxExecDevices: shard pointers go through device memory, 4 tables of ndev pointers
  // (caller's sources, caller's destinations, the two workspace regions) behind the descriptors, refreshed on
  // every call
  size_t ptr_tables_off = 0;
  size_t device_bytes = 0;             // descriptors plus pointer tables
  // device copy of the descriptors (after prepare)
  std::mutex mu;
  std::atomic<bool> prepared{false};
  int device = -1;
  char* dev_blob = nullptr;
};

namespace {

int64_t align_up(int64_t v, int64_t a) { return (v + a - 1) / a * a; }

redist_status to_status(Status s) { return static_cast<redist_status>(s); }

bool read_type(const redist_type* t, TypeSpec* out) {
  if (!t || t->rank < 1 || t->rank > REDIST_MAX_RANK || !t->global_shape || !t->n_axes_of_dim) return false;
  out->gshape.assign(t->global_shape, t->global_shape + t->rank);
  out->axes.assign(t->rank, {});
  int pos = 0;
  for (int k = 0; k < t->rank; ++k) {
    int n = t->n_axes_of_dim[k];
    if (n < 0 || n > 64) return false;
    if (n > 0 && !t->axes_flat) return false;
    for (int a = 0; a < n; ++a) out->axes[k].push_back(t->axes_flat[pos++]);
  }
  return true;
}

}  // namespace

extern "C" {

static int64_t predicted_ns_of(const redist_plan* p) {
  int64_t ns = 0;
  for (const CopyOp& op : p->ops) {
    const int64_t bytes = op.cell.enabled ? op.cell.bytes_read + op.cell.bytes_written
                          : op.row.enabled ? op.row.bytes_read + op.row.bytes_written : op.bytes_read + op.bytes_written;
    ns += p->launch_latency_ns + bytes / std::max<int64_t>(1, p->sustained_gbs);   // 1 GB/s = 1 byte per ns
  }
  return ns;
}

static BuildOptions read_options(const redist_options* o, int64_t* latency) {
  BuildOptions b;
  *latency = 0;
  if (!o) return b;
  b.merge_runs = o->merge_runs != 0;
  b.fold_permute = o->fold_permute != 0;
  b.lds_staging = o->lds_staging != 0;
  b.row_dst_order = o->lds_staging != 2;
  b.span_form = o->span_form != 0;
  b.dest_major = o->dest_major != 0;
  b.unroll = o->unroll;
  b.dest_major_min_bytes = o->dest_major_min_bytes;
  if (o->max_grid) b.max_grid = o->max_grid;
  b.dm_fanout = o->dest_major_fanout;
  b.cell_form = o->cell_form;
  b.siblings = o->sibling_sources != 0;
  if (o->sibling_sources > 1) b.sib_max_run = o->sibling_sources;
  *latency = o->step_latency_elems < 0 ? 0 : o->step_latency_elems;
  return b;
}

static redist_status plan_create_impl(const redist_mesh* mesh, const redist_type* src, const redist_type* dst,
                                      int32_t elem_size, uint32_t mode, const redist_options* options,
                                      redist_plan** out) {
  if (!mesh || !src || !dst || !out) return REDIST_ERR_NULL;
  if (options && options->struct_size != sizeof(redist_options)) return REDIST_ERR_BAD_ARG;
  if (mesh->n_axes < 1 || mesh->n_axes > 64 || !mesh->axis_size) return REDIST_ERR_BAD_MESH;
  if (src->rank < 1 || dst->rank < 1 || src->rank > REDIST_MAX_RANK || dst->rank > REDIST_MAX_RANK)
    return REDIST_ERR_ILL_FORMED;
  if (!src->global_shape || !dst->global_shape || !src->n_axes_of_dim || !dst->n_axes_of_dim) return REDIST_ERR_NULL;
  std::vector<int64_t> sizes(mesh->axis_size, mesh->axis_size + mesh->n_axes);
  TypeSpec ts, td;
  if (!read_type(src, &ts) || !read_type(dst, &td)) return REDIST_ERR_ILL_FORMED;
  if (src->rank != dst->rank) {
    // still report ill-formed inputs first; otherwise the global types differ
    return REDIST_ERR_GLOBAL_MISMATCH;
  }
  if (mode == REDIST_MODE_AUTO) {
    // both candidates; the stepwise one with a latency term in its search: one launch is worth
    // launch latency x sustained rate bytes, i.e. that many bytes / (2 x elem_size x devices) elements per device
    redist_options o;
    if (options) o = *options; else redist_options_init(&o);
    int64_t ndev = 1;
    for (int64_t k : sizes) ndev *= std::max<int64_t>(1, k);
    const int64_t lat_ns = o.launch_latency_ns > 0 ? o.launch_latency_ns : 3000;
    const int64_t gbs = o.sustained_gbs > 0 ? o.sustained_gbs : 5500;
    if (o.step_latency_elems == 0 && elem_size > 0) o.step_latency_elems = lat_ns * gbs / (2 * elem_size * ndev);
    redist_plan *stepwise = nullptr, *fused = nullptr;
    redist_status e = plan_create_impl(mesh, src, dst, elem_size, REDIST_MODE_STEPWISE, &o, &stepwise);
    if (e != REDIST_OK) return e;
    e = plan_create_impl(mesh, src, dst, elem_size, REDIST_MODE_FUSED, &o, &fused);
    if (e != REDIST_OK) { redist_plan_destroy(stepwise); return e; }
    const bool keep_stepwise = predicted_ns_of(stepwise) <= predicted_ns_of(fused);
    redist_plan_destroy(keep_stepwise ? fused : stepwise);
    *out = keep_stepwise ? stepwise : fused;
    return REDIST_OK;
  }
  std::unique_ptr<redist_plan> p(new redist_plan());
  int64_t latency = 0;
  p->opt = read_options(options, &latency);
  if (options && options->launch_latency_ns > 0) p->launch_latency_ns = options->launch_latency_ns;
  if (options && options->sustained_gbs > 0) p->sustained_gbs = options->sustained_gbs;
  Status s = make_plan(sizes, ts, td, elem_size, (int)mode, latency, &p->core);
  if (s != kOk) return to_status(s);
  const PlanCore& pc = p->core;
  const BuildOptions& opt = p->opt;
  const int B = pc.elem_size, r = pc.rank, nd = pc.ndev;

  // one copy op per launch; an empty step list (src == dst) is carried out as an identity copy
  const std::vector<int64_t>* cs = &pc.shape_src;
  const std::vector<int64_t>* os = &pc.offs_src;
  bool ok = true;
  if (pc.steps.empty()) {
    CopyOp op;
    ok = build_copy_op(kAllPermute, nd, r, B, pc.shape_src, pc.offs_src, pc.shape_dst, pc.offs_dst, opt, &op);
    p->ops.push_back(std::move(op));  // identical tiles on both sides: never a row-complete op
  }
  // Which steps share a launch (stepwise mode; the naive baseline stays literal).  A step is carried out from the
  // device tables before and after it, and the tables before a group's first and after its last step describe the
  // whole group, so the intermediate types inside a group never exist in memory:
  //  - a run of consecutive dynslices, or of consecutive allgathers, is one launch (a slice of a slice is a slice;
  //    gathering dim after dim reads one tile into every shard that ends up holding it);
  //  - a run of dynslices shares the launch of what follows it: slicing is local (Sec. 4.1, it needs no
  //    communication), so the next collective simply reads the part of each tile that the slice keeps;
  //  - the allpermute shares the launch of the alltoall in front of it, else of the allgathers after it: the
  //    normal form has at most one, placed between the two (Eq. (6)-(7), Sec. 7.3), and on a virtual mesh it moves
  //    whole tiles, i.e. it only says which shard the neighbouring collective writes to (or reads from).
  // Collectives that communicate (alltoall; allgather after another kind) stay one launch each.  A launch holds
  // its first input and its last output, at most source tile + target tile, which the caller's buffers occupy
  // for the whole call anyway.
  const bool merge_runs = pc.mode == REDIST_MODE_STEPWISE && opt.merge_runs;
  const bool fold_permute = merge_runs && opt.fold_permute;
  const size_t n_steps = pc.steps.size();
  auto kind_at = [&](size_t k) { return k < n_steps ? pc.steps[k].kind : -1; };
  auto end_of_run = [&](size_t from) {
    size_t l = from;
    if (pc.steps[from].kind == kDynSlice || pc.steps[from].kind == kAllGather)
      while (l + 1 < n_steps && pc.steps[l + 1].kind == pc.steps[from].kind) ++l;
    return l;
  };
  for (size_t k = 0; k < n_steps;) {
    size_t last = k, main = k;   // main: the step whose kind names the kernel
    if (merge_runs) {
      last = end_of_run(k);
      if (pc.steps[k].kind == kDynSlice && last + 1 < n_steps) {
        main = last + 1;
        last = end_of_run(main);
      }
      if (fold_permute) {
        if (kind_at(main) == kAllToAll && kind_at(last + 1) == kAllPermute) {
          ++last;
        } else if (kind_at(main) == kAllPermute && kind_at(last + 1) == kAllGather) {
          main = last + 1;
          last = end_of_run(main);
        }
      }
    }
    const Step& st = pc.steps[last];
    CopyOp op;
    ok = ok && build_copy_op(pc.steps[main].kind, nd, r, B, *cs, *os, st.shape_after, st.offs_after, opt, &op);
    if (ok) build_row_op(nd, r, B, *cs, *os, st.shape_after, st.offs_after, opt, &op.row);
    if (ok) {
      // cells take over where the body chosen so far moves short stretches
      OtherBody other;
      if (op.row.enabled) {
        other.stretch = op.row.min_stretch;
        other.strong = op.row.vn == 16;
        other.dest_major = op.row.dest_major;
      } else {
        other.stretch = INT64_MAX;
        for (const DevBox& bx : op.boxes) other.stretch = std::min<int64_t>(other.stretch, (int64_t)bx.run_vecs * op.vec_bytes);
        other.dest_major = op.dest_major;
      }
      build_cell_op(nd, r, B, *cs, *os, st.shape_after, st.offs_after, opt, other, &op.cell);
    }
    p->ops.push_back(std::move(op));
    p->op_last_step.push_back((int)last);
    cs = &st.shape_after;
    os = &st.offs_after;
    k = last + 1;
  }
  if (!ok) return REDIST_ERR_UNSUPPORTED;

  // workspace: intermediates ping-pong between two regions (odd / even step index)
  size_t n_ops = p->ops.size();
  p->shard_stride.assign(n_ops, 0);
  p->region_off.assign(n_ops, 0);
  int64_t region_size[2] = {0, 0};
  for (size_t k = 0; k + 1 < n_ops; ++k) {
    int64_t bytes = align_up(product(pc.steps[(size_t)p->op_last_step[k]].shape_after) * B, 256);
    p->shard_stride[k] = bytes;
    region_size[k & 1] = std::max(region_size[k & 1], bytes * nd);
  }
  for (size_t k = 0; k + 1 < n_ops; ++k) p->region_off[k] = (k & 1) ? region_size[0] : 0;
  p->workspace_bytes = region_size[0] + region_size[1];

  // host image of the descriptors
  size_t total = 0;
  auto reserve = [&](std::vector<size_t>* offs, size_t bytes) {
    offs->push_back(total);
    total += (size_t)align_up((int64_t)bytes, 256);
  };
  for (const CopyOp& op : p->ops) {
    reserve(&p->boxes_off, op.boxes.size() * sizeof(DevBox));
    reserve(&p->list_off, op.dst_list.size() * sizeof(int32_t));
    reserve(&p->rbox_off, op.row.boxes.size() * sizeof(DevRowBox));
    reserve(&p->rpiece_off, op.row.pieces.size() * sizeof(DevPiece));
    reserve(&p->rlist_off, op.row.dev_list.size() * sizeof(int32_t));
    reserve(&p->cbox_off, op.cell.boxes.size() * sizeof(DevCellBox));
    reserve(&p->clist_off, op.cell.dev_list.size() * sizeof(int32_t));
  }
  p->blob.assign(total, 0);
  auto put = [&](size_t off, const void* from, size_t bytes) {
    if (bytes) std::memcpy(p->blob.data() + off, from, bytes);
  };
  for (size_t k = 0; k < n_ops; ++k) {
    const CopyOp& op = p->ops[k];
    put(p->boxes_off[k], op.boxes.data(), op.boxes.size() * sizeof(DevBox));
    put(p->list_off[k], op.dst_list.data(), op.dst_list.size() * sizeof(int32_t));
    put(p->rbox_off[k], op.row.boxes.data(), op.row.boxes.size() * sizeof(DevRowBox));
    put(p->rpiece_off[k], op.row.pieces.data(), op.row.pieces.size() * sizeof(DevPiece));
    put(p->rlist_off[k], op.row.dev_list.data(), op.row.dev_list.size() * sizeof(int32_t));
    put(p->cbox_off[k], op.cell.boxes.data(), op.cell.boxes.size() * sizeof(DevCellBox));
    put(p->clist_off[k], op.cell.dev_list.data(), op.cell.dev_list.size() * sizeof(int32_t));
  }
  p->ptr_tables_off = total;
  if (nd > kMaxExecDevices) total += (size_t)align_up((int64_t)(4 * (size_t)nd * sizeof(void*)), 256);
  p->device_bytes = total;
  *out = p.release();
  return REDIST_OK;
}

// Nothing may throw across the C boundary: allocation failures become a status.
redist_status redist_plan_create(const redist_mesh* mesh, const redist_type* src, const redist_type* dst,
                                 int32_t elem_size, uint32_t mode, redist_plan** out) {
  try {
    return plan_create_impl(mesh, src, dst, elem_size, mode, nullptr, out);
  } catch (...) {
    return REDIST_ERR_INTERNAL;
  }
}

void redist_options_init(redist_options* o) {
  if (!o) return;
  const BuildOptions d;
  std::memset(o, 0, sizeof(*o));
  o->struct_size = (uint32_t)sizeof(redist_options);
  o->merge_runs = d.merge_runs;
  o->fold_permute = d.fold_permute;
  o->lds_staging = d.lds_staging;
  o->span_form = d.span_form;
  o->dest_major = d.dest_major;
  o->unroll = d.unroll;
  o->dest_major_min_bytes = d.dest_major_min_bytes;
  o->max_grid = d.max_grid;
  o->step_latency_elems = 0;
  o->launch_latency_ns = 3000;
  o->sustained_gbs = 5500;
  o->cell_form = d.cell_form;
  o->sibling_sources = d.siblings;
  o->dest_major_fanout = 0;
}

void redist_plan_destroy(redist_plan* plan) {
  if (!plan) return;
  if (plan->refs.fetch_sub(1) != 1) return;   // still referenced (by the cache or by another holder of a cached plan)
  if (plan->dev_blob) (void)hipFree(plan->dev_blob);
  delete plan;
}

// ---- plan cache: equal arguments share one plan ----
namespace {
struct PlanCache {
  std::mutex mu;
  std::map<std::vector<int64_t>, redist_plan*> plans;   // key = every argument of redist_plan_create, flattened
  std::deque<std::vector<int64_t>> order;               // insertion order, oldest first
  size_t capacity = 1024;
};
PlanCache& plan_cache() {
  static PlanCache c;
  return c;
}
bool flatten_key(const redist_mesh* mesh, const redist_type* src, const redist_type* dst, int32_t elem_size, uint32_t mode,
                 const redist_options* options, std::vector<int64_t>* key) {
  if (!mesh || !src || !dst || mesh->n_axes < 1 || mesh->n_axes > 64 || !mesh->axis_size) return false;
  if (options && options->struct_size != sizeof(redist_options)) return false;
  int64_t latency = 0;
  const BuildOptions o = read_options(options, &latency);
  key->assign({(int64_t)elem_size, (int64_t)mode, (int64_t)mesh->n_axes});
  // the options are part of a plan's identity
  key->insert(key->end(), {(int64_t)o.merge_runs, (int64_t)o.fold_permute, (int64_t)o.lds_staging, (int64_t)o.span_form,
                           (int64_t)o.dest_major, (int64_t)o.unroll, o.dest_major_min_bytes, (int64_t)o.max_grid, latency,
                           (int64_t)(options ? options->launch_latency_ns : 3000),
                           (int64_t)(options ? options->sustained_gbs : 5500), (int64_t)o.dm_fanout, (int64_t)o.cell_form, (int64_t)o.siblings, o.sib_max_run, (int64_t)o.row_dst_order});
  key->insert(key->end(), mesh->axis_size, mesh->axis_size + mesh->n_axes);
  for (const redist_type* t : {src, dst}) {
    TypeSpec ts;
    if (!read_type(t, &ts)) return false;
    key->push_back(t->rank);
    for (int k = 0; k < t->rank; ++k) {
      key->push_back(ts.gshape[(size_t)k]);
      key->push_back((int64_t)ts.axes[(size_t)k].size());
      key->insert(key->end(), ts.axes[(size_t)k].begin(), ts.axes[(size_t)k].end());
    }
  }
  return true;
}
}  // namespace

static redist_status plan_create_cached_impl(const redist_mesh* mesh, const redist_type* src, const redist_type* dst,
                                             int32_t elem_size, uint32_t mode, const redist_options* options,
                                             redist_plan** out) {
  if (!out) return REDIST_ERR_NULL;
  std::vector<int64_t> key;
  if (!flatten_key(mesh, src, dst, elem_size, mode, options, &key))
    return plan_create_impl(mesh, src, dst, elem_size, mode, options, out);   // reports what is wrong with the arguments
  PlanCache& c = plan_cache();
  {
    std::lock_guard<std::mutex> lock(c.mu);
    auto it = c.plans.find(key);
    if (it != c.plans.end()) {
      it->second->refs.fetch_add(1);
      *out = it->second;
      return REDIST_OK;
    }
  }
  // Synthesis runs outside the lock (usually a fraction of a millisecond, but seconds at the limits the boundary
  // accepts: rank 8 on 4096 devices); two threads that miss on the same key both plan, the second one to come
  // back drops its plan and takes the cached one.
  redist_plan* p = nullptr;
  redist_status s = plan_create_impl(mesh, src, dst, elem_size, mode, options, &p);
  if (s != REDIST_OK) return s;
  std::lock_guard<std::mutex> lock(c.mu);
  auto it = c.plans.find(key);
  if (it != c.plans.end()) {
    redist_plan_destroy(p);
    it->second->refs.fetch_add(1);
    *out = it->second;
    return REDIST_OK;
  }
  while (c.plans.size() >= c.capacity && !c.order.empty()) {   // drop the oldest entry; its holders keep it alive
    auto old = c.plans.find(c.order.front());
    c.order.pop_front();
    if (old != c.plans.end()) {
      redist_plan* victim = old->second;
      c.plans.erase(old);
      redist_plan_destroy(victim);
    }
  }
  p->refs.fetch_add(1);   // the cache's own reference
  c.plans.emplace(key, p);
  c.order.push_back(std::move(key));
  *out = p;
  return REDIST_OK;
}

redist_status redist_plan_create_cached(const redist_mesh* mesh, const redist_type* src, const redist_type* dst,
                                        int32_t elem_size, uint32_t mode, redist_plan** out) {
  try {
    return plan_create_cached_impl(mesh, src, dst, elem_size, mode, nullptr, out);
  } catch (...) {
    return REDIST_ERR_INTERNAL;
  }
}

redist_status redist_plan_create_ex(const redist_mesh* mesh, const redist_type* src, const redist_type* dst,
                                    int32_t elem_size, uint32_t mode, const redist_options* opt, int32_t cached,
                                    redist_plan** out) {
  try {
    return cached ? plan_create_cached_impl(mesh, src, dst, elem_size, mode, opt, out)
                  : plan_create_impl(mesh, src, dst, elem_size, mode, opt, out);
  } catch (...) {
    return REDIST_ERR_INTERNAL;
  }
}

void redist_plan_cache_clear(void) {
  PlanCache& c = plan_cache();
  std::lock_guard<std::mutex> lock(c.mu);
  for (auto& kv : c.plans) redist_plan_destroy(kv.second);
  c.plans.clear();
  c.order.clear();
}

int32_t redist_plan_cache_size(void) {
  PlanCache& c = plan_cache();
  std::lock_guard<std::mutex> lock(c.mu);
  return (int32_t)c.plans.size();
}

int32_t redist_plan_num_devices(const redist_plan* p) { return p ? p->core.ndev : -1; }
int32_t redist_plan_rank(const redist_plan* p) { return p ? p->core.rank : -1; }
int32_t redist_plan_mode(const redist_plan* p) { return p ? p->core.mode : -1; }
int32_t redist_plan_num_steps(const redist_plan* p) { return p ? (int32_t)p->core.steps.size() : -1; }

redist_status redist_plan_step(const redist_plan* p, int32_t k, int32_t* kind, int32_t* dim_i, int32_t* dim_j,
                               int64_t* factor, int64_t* local_shape_after) {
  if (!p) return REDIST_ERR_NULL;
  if (k < 0 || k >= (int32_t)p->core.steps.size()) return REDIST_ERR_BAD_ARG;
  const Step& st = p->core.steps[(size_t)k];
  if (kind) *kind = st.kind;
  if (dim_i) *dim_i = st.dim_i;
  if (dim_j) *dim_j = st.dim_j;
  if (factor) *factor = st.factor;
  if (local_shape_after) std::memcpy(local_shape_after, st.shape_after.data(), sizeof(int64_t) * st.shape_after.size());
  return REDIST_OK;
}

redist_status redist_plan_step_offsets(const redist_plan* p, int32_t k, int64_t* out) {
  if (!p || !out) return REDIST_ERR_NULL;
  if (k < -1 || k >= (int32_t)p->core.steps.size()) return REDIST_ERR_BAD_ARG;
  const std::vector<int64_t>& t = k < 0 ? p->core.offs_src : p->core.steps[(size_t)k].offs_after;
  std::memcpy(out, t.data(), sizeof(int64_t) * t.size());
  return REDIST_OK;
}

redist_status redist_plan_step_peers(const redist_plan* p, int32_t k, int32_t* out) {
  if (!p || !out) return REDIST_ERR_NULL;
  if (k < 0 || k >= (int32_t)p->core.steps.size()) return REDIST_ERR_BAD_ARG;
  const Step& st = p->core.steps[(size_t)k];
  if (st.kind == kFused) return REDIST_ERR_BAD_ARG;
  std::memcpy(out, st.peers.data(), sizeof(int32_t) * st.peers.size());
  return REDIST_OK;
}

int64_t redist_plan_cost_elems(const redist_plan* p) { return p ? p->core.cost : -1; }
int64_t redist_plan_weak_cost_elems(const redist_plan* p) { return p ? p->core.weak_cost : -1; }
int64_t redist_plan_height_elems(const redist_plan* p) { return p ? p->core.height : -1; }
int64_t redist_plan_bound_elems(const redist_plan* p) { return p ? p->core.bound : -1; }

int64_t redist_plan_peak_live_bytes_per_shard(const redist_plan* p) {
  if (!p) return -1;
  const PlanCore& pc = p->core;
  int64_t L = product(pc.shape_src), peak = 0;
  if (pc.steps.empty()) peak = 2 * L;
  for (int last : p->op_last_step) {   // per launch: its source and its destination are live together
    int64_t Ln = product(pc.steps[(size_t)last].shape_after);
    peak = std::max(peak, L + Ln);
    L = Ln;
  }
  return peak * pc.elem_size;
}

int64_t redist_plan_workspace_bytes(const redist_plan* p) { return p ? p->workspace_bytes : -1; }
int64_t redist_plan_predicted_ns(const redist_plan* p) { return p ? predicted_ns_of(p) : -1; }
int32_t redist_plan_search_limits_hit(const redist_plan* p) { return p ? (int32_t)p->core.limits_hit : -1; }

int64_t redist_plan_footprint_bytes_per_shard(const redist_plan* p) {
  if (!p) return -1;
  const PlanCore& pc = p->core;
  return (product(pc.shape_src) + product(pc.shape_dst)) * pc.elem_size + p->workspace_bytes / pc.ndev;
}

redist_status redist_plan_op_output(const redist_plan* p, int32_t k, int64_t* region_off, int64_t* shard_stride) {
  if (!p) return REDIST_ERR_NULL;
  if (k < 0 || (size_t)k + 1 >= p->ops.size()) return REDIST_ERR_BAD_ARG;
  if (region_off) *region_off = p->region_off[(size_t)k];
  if (shard_stride) *shard_stride = p->shard_stride[(size_t)k];
  return REDIST_OK;
}

int64_t redist_plan_algorithmic_bytes(const redist_plan* p, int32_t which) {
  if (!p) return -1;
  const PlanCore& pc = p->core;
  switch (which) {
    case REDIST_BYTES_READ_MIN: return product(pc.gshape) * pc.elem_size;
    case REDIST_BYTES_READ_LOGICAL:
    case REDIST_BYTES_WRITE: return (int64_t)pc.ndev * product(pc.shape_dst) * pc.elem_size;
    case REDIST_BYTES_MOVED_BY_PLAN: {
      int64_t b = 0;
      for (const CopyOp& op : p->ops)
        b += op.cell.enabled ? op.cell.bytes_read + op.cell.bytes_written
             : op.row.enabled ? op.row.bytes_read + op.row.bytes_written : op.bytes_read + op.bytes_written;
      return b;
    }
    default: return -1;
  }
}

const char* redist_plan_step_kernel(const redist_plan* p, int32_t k) {
  if (!p) return "";
  if (k < 0 || k >= (int32_t)p->ops.size()) return "";
  const CopyOp& op = p->ops[(size_t)k];
  return op.cell.enabled ? cell_kernel_name_of(op.kind) : op.row.enabled ? row_kernel_name_of(op.kind) : kernel_name_of(op.kind);
}

int32_t redist_plan_num_ops(const redist_plan* p) { return p ? (int32_t)p->ops.size() : -1; }

int32_t redist_plan_op_last_step(const redist_plan* p, int32_t k) {
  if (!p || k < 0 || k >= (int32_t)p->op_last_step.size()) return -1;
  return p->op_last_step[(size_t)k];
}

redist_status redist_plan_op_info(const redist_plan* p, int32_t k, redist_op_info* out) {
  if (!p || !out) return REDIST_ERR_NULL;
  if (k < 0 || k >= (int32_t)p->ops.size()) return REDIST_ERR_BAD_ARG;
  const CopyOp& op = p->ops[(size_t)k];
  const PlanCore& pc = p->core;
  redist_op_info o{};
  o.kind = op.kind;
  o.n_boxes = (int32_t)op.boxes.size();
  o.n_dst_list = (int32_t)op.dst_list.size();
  o.n_outer = op.n_outer;
  o.vec_bytes = op.vec_bytes;
  o.tc = op.tc;
  o.tr = op.tr;
  o.tc_magic = op.tc_magic;
  o.tc_shift = op.tc_shift;
  o.n_tiles = op.n_tiles;
  o.tiles_per_box = op.tiles_per_box;
  o.unroll = op.unroll;
  o.nontemporal = op.nontemporal ? 1 : 0;
  o.dest_major = op.dest_major ? 1 : 0;
  o.chunk_tiles = op.chunk_tiles;
  o.src_tiles = op.src_tiles;
  o.dm_count = op.dm_count;
  o.dm_magic = op.dm_magic;
  o.dm_shift = op.dm_shift;
  o.max_grid = op.max_grid;
  o.dm_fanout = op.dm_fanout;
  o.dm_groups = op.dm_groups;
  o.sib_count = op.sib_count; o.sib_magic = op.sib_magic; o.sib_shift = op.sib_shift; o.sib_inner_log2 = op.sib_inner_log2;
  o.tpb_magic = op.tpb_magic;
  o.tpb_shift = op.tpb_shift;
  for (int t = 0; t < kMaxOuter; ++t) { o.sstride[t] = op.sstride[t]; o.dstride[t] = op.dstride[t]; }
  const size_t n_ops = p->ops.size();
  o.src_shard_bytes = product(k == 0 ? pc.shape_src : pc.steps[(size_t)p->op_last_step[(size_t)k - 1]].shape_after) * pc.elem_size;
  o.dst_shard_bytes = product((size_t)k + 1 == n_ops ? pc.shape_dst : pc.steps[(size_t)p->op_last_step[(size_t)k]].shape_after) * pc.elem_size;
  *out = o;
  return REDIST_OK;
}

redist_status redist_plan_op_tables(const redist_plan* p, int32_t k, redist_box* boxes, int32_t* dst_list) {
  if (!p) return REDIST_ERR_NULL;
  if (k < 0 || k >= (int32_t)p->ops.size()) return REDIST_ERR_BAD_ARG;
  const CopyOp& op = p->ops[(size_t)k];
  static_assert(sizeof(redist_box) == sizeof(DevBox), "public and internal box layouts must agree");
  if (boxes && !op.boxes.empty()) std::memcpy(boxes, op.boxes.data(), op.boxes.size() * sizeof(DevBox));
  if (dst_list && !op.dst_list.empty())
    std::memcpy(dst_list, op.dst_list.data(), op.dst_list.size() * sizeof(int32_t));
  return REDIST_OK;
}

redist_status redist_plan_op_row_info(const redist_plan* p, int32_t k, redist_row_info* out) {
  if (!p || !out) return REDIST_ERR_NULL;
  if (k < 0 || k >= (int32_t)p->ops.size()) return REDIST_ERR_BAD_ARG;
  const RowOp& op = p->ops[(size_t)k].row;
  const PlanCore& pc = p->core;
  redist_row_info o{};
  o.enabled = op.enabled ? 1 : 0;
  o.dir = op.dir; o.n_outer = op.n_outer; o.w_log2 = op.w_log2; o.n_log2 = op.n_log2; o.r_log2 = op.r_log2;
  o.vn = op.vn; o.n_pieces = op.n_pieces; o.narrow_count = op.narrow_count;
  o.n_boxes = (int32_t)op.boxes.size();
  o.n_pieces_total = (int32_t)op.pieces.size();
  o.n_dev_list = (int32_t)op.dev_list.size();
  o.n_tiles = op.n_tiles; o.tiles_per_box = op.tiles_per_box; o.tpb_magic = op.tpb_magic; o.tpb_shift = op.tpb_shift;
  o.general = op.general ? 1 : 0;
  o.w_bytes = op.w_bytes; o.n_bytes = op.n_bytes; o.pitch = op.pitch;
  o.cpn = op.cpn; o.cpn_magic = op.cpn_magic; o.cpn_shift = op.cpn_shift;
  o.wpr = op.wpr; o.wpr_magic = op.wpr_magic; o.wpr_shift = op.wpr_shift;
  o.vw = op.vw;
  o.span = op.span ? 1 : 0; o.gran = op.gran; o.chunk_dims = op.chunk_dims; o.rpt = op.rpt; o.rpt_magic = op.rpt_magic; o.rpt_shift = op.rpt_shift; o.mct = op.mct; o.slot = op.slot;
  o.cbw = op.cbw; o.cbw_magic = op.cbw_magic; o.cbw_shift = op.cbw_shift;
  o.nbm = op.nbm; o.nbm_magic = op.nbm_magic; o.nbm_shift = op.nbm_shift;
  for (int t = 0; t < kMaxOuter; ++t) { o.wstride[t] = op.enabled ? op.wstride[t] : 0; o.nstride[t] = op.enabled ? op.nstride[t] : 0; }
  o.dest_major = op.dest_major ? 1 : 0;
  o.dm_count = op.dm_count; o.dm_magic = op.dm_magic; o.dm_shift = op.dm_shift;
  o.chunk_tiles = op.chunk_tiles; o.src_tiles = op.src_tiles;
  o.max_grid = op.max_grid;
  o.dm_fanout = op.dm_fanout; o.dm_groups = op.dm_groups;
  const size_t n_ops = p->ops.size();
  o.src_shard_bytes = product(k == 0 ? pc.shape_src : pc.steps[(size_t)p->op_last_step[(size_t)k - 1]].shape_after) * pc.elem_size;
  o.dst_shard_bytes = product((size_t)k + 1 == n_ops ? pc.shape_dst : pc.steps[(size_t)p->op_last_step[(size_t)k]].shape_after) * pc.elem_size;
  *out = o;
  return REDIST_OK;
}

redist_status redist_plan_op_row_tables(const redist_plan* p, int32_t k, redist_row_box* boxes, redist_piece* pieces,
                                        int32_t* dev_list) {
  if (!p) return REDIST_ERR_NULL;
  if (k < 0 || k >= (int32_t)p->ops.size()) return REDIST_ERR_BAD_ARG;
  const RowOp& op = p->ops[(size_t)k].row;
  static_assert(sizeof(redist_row_box) == sizeof(DevRowBox) && sizeof(redist_piece) == sizeof(DevPiece),
                "public and internal row descriptor layouts must agree");
  if (boxes && !op.boxes.empty()) std::memcpy(boxes, op.boxes.data(), op.boxes.size() * sizeof(DevRowBox));
  if (pieces && !op.pieces.empty()) std::memcpy(pieces, op.pieces.data(), op.pieces.size() * sizeof(DevPiece));
  if (dev_list && !op.dev_list.empty()) std::memcpy(dev_list, op.dev_list.data(), op.dev_list.size() * sizeof(int32_t));
  return REDIST_OK;
}

redist_status redist_plan_op_cell_info(const redist_plan* p, int32_t k, redist_cell_info* out) {
  if (!p || !out) return REDIST_ERR_NULL;
  if (k < 0 || (size_t)k >= p->ops.size()) return REDIST_ERR_BAD_ARG;
  const CellOp& op = p->ops[(size_t)k].cell;
  redist_cell_info o{};
  o.enabled = op.enabled ? 1 : 0;
  if (op.enabled) {
    o.n_outer = op.n_outer; o.n_cell = op.n_cell; o.ps = op.ps; o.pd = op.pd; o.rep = op.rep;
    o.vs = op.vs; o.vd = op.vd; o.gran = op.gran; o.base_first = op.base_first;
    o.rows_per_tile = op.rows_per_tile; o.src_row_bytes = op.src_row_bytes; o.dst_row_bytes = op.dst_row_bytes;
    o.part_pitch = op.part_pitch; o.drow_gran = op.drow_gran;
    for (int i = 0; i < kMaxCellDims; ++i) {
      o.dext[i] = op.dext[i]; o.piece[i] = op.piece[i]; o.lds_step[i] = op.lds_step[i]; o.part_step[i] = op.part_step[i];
    }
    for (int i = 0; i < kMaxOuter; ++i) { o.sstride[i] = op.sstride[i]; o.dstride[i] = op.dstride[i]; }
    o.n_boxes = (int32_t)op.boxes.size(); o.n_list = (int32_t)op.dev_list.size();
    o.n_tiles = op.n_tiles; o.max_grid = op.max_grid;
    o.bytes_read = op.bytes_read; o.bytes_written = op.bytes_written; o.min_stretch = op.min_stretch;
    o.spv = op.spv; o.spv_magic = op.spv_magic; o.spv_shift = op.spv_shift;
    o.dpv = op.dpv; o.dpv_magic = op.dpv_magic; o.dpv_shift = op.dpv_shift;
    o.drg_magic = op.drg_magic; o.drg_shift = op.drg_shift;
    for (int i = 0; i < kMaxCellDims; ++i) {
      o.dext_magic[i] = op.dext_magic[i]; o.dext_shift[i] = op.dext_shift[i];
      o.piece_magic[i] = op.piece_magic[i]; o.piece_shift[i] = op.piece_shift[i];
    }
    o.tiles_per_box = op.tiles_per_box; o.tpb_magic = op.tpb_magic; o.tpb_shift = op.tpb_shift;
  }
  *out = o;
  return REDIST_OK;
}

redist_status redist_plan_op_cell_tables(const redist_plan* p, int32_t k, redist_cell_box* boxes, int32_t* dev_list) {
  if (!p) return REDIST_ERR_NULL;
  if (k < 0 || (size_t)k >= p->ops.size()) return REDIST_ERR_BAD_ARG;
  const CellOp& op = p->ops[(size_t)k].cell;
  static_assert(sizeof(redist_cell_box) == sizeof(DevCellBox), "public and internal cell descriptor layouts must agree");
  if (boxes && !op.boxes.empty()) std::memcpy(boxes, op.boxes.data(), op.boxes.size() * sizeof(DevCellBox));
  if (dev_list && !op.dev_list.empty()) std::memcpy(dev_list, op.dev_list.data(), op.dev_list.size() * sizeof(int32_t));
  return REDIST_OK;
}

static redist_status plan_prepare_impl(redist_plan* p) {
  if (!p) return REDIST_ERR_NULL;
  std::lock_guard<std::mutex> lock(p->mu);
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess) return REDIST_ERR_HIP;
  if (p->prepared && p->device == dev) return REDIST_OK;
  if (p->prepared) return REDIST_ERR_UNSUPPORTED;  // a plan is bound to the device it was prepared on
  const size_t total = p->device_bytes;
  void* blob = nullptr;
  if (hipMalloc(&blob, total ? total : 256) != hipSuccess) return REDIST_ERR_HIP;
  if (!p->blob.empty() && hipMemcpy(blob, p->blob.data(), p->blob.size(), hipMemcpyHostToDevice) != hipSuccess) {
    (void)hipFree(blob);
    return REDIST_ERR_HIP;
  }
  p->dev_blob = static_cast<char*>(blob);
  p->device = dev;
  p->prepared = true;
  return REDIST_OK;
}

redist_status redist_plan_prepare(redist_plan* p) {
  try {
    return plan_prepare_impl(p);
  } catch (...) {
    return REDIST_ERR_INTERNAL;
  }
}

// Enqueue launches [op_begin, op_end) of the plan; `desc` is the device copy of the plan's descriptor image.
static redist_status enqueue_ops(const redist_plan* p, char* desc, const void* const* src_shards, void* const* dst_shards,
                                 void* workspace, void* hip_stream, size_t op_begin, size_t op_end) {
  const int nd = p->core.ndev;
  const size_t n_ops = p->ops.size();
  const bool reads_src = op_begin == 0, writes_dst = op_end == n_ops;
  const bool uses_ws = n_ops > 1;   // every launch of a multi-launch plan reads or writes an intermediate
  if (reads_src && !src_shards) return REDIST_ERR_NULL;
  if (writes_dst && !dst_shards) return REDIST_ERR_NULL;
  if (uses_ws && p->workspace_bytes > 0 && !workspace) return REDIST_ERR_WORKSPACE;
  if (workspace && (reinterpret_cast<uintptr_t>(workspace) & 255u)) return REDIST_ERR_BAD_ARG;
  for (int d = 0; d < nd; ++d) {
    if ((reads_src && !src_shards[d]) || (writes_dst && !dst_shards[d])) return REDIST_ERR_NULL;
    if ((reads_src && (reinterpret_cast<uintptr_t>(src_shards[d]) & 15u)) ||
        (writes_dst && (reinterpret_cast<uintptr_t>(dst_shards[d]) & 15u)))
      return REDIST_ERR_BAD_ARG;
  }
  const bool big = nd > kMaxExecDevices;
  PtrTable user_src{}, user_dst{};
  // big meshes: device memory behind the descriptors holds [sources | destinations | workspace intermediates of
  // odd / even steps]
  void** dev_tables = big ? reinterpret_cast<void**>(desc + p->ptr_tables_off) : nullptr;
  if (!big) {
    for (int d = 0; d < nd; ++d) {
      if (reads_src) user_src.p[d] = const_cast<void*>(src_shards[d]);
      if (writes_dst) user_dst.p[d] = dst_shards[d];
    }
  } else {
    // Pointer tables travel through plan-owned device memory, written by kernels ordered on the caller's
    // stream; executing one such plan on two streams at once would race on them.
    if ((reads_src && launch_ptr_table(src_shards, nd, dev_tables, hip_stream) != 0) ||
        (writes_dst && launch_ptr_table(dst_shards, nd, dev_tables + nd, hip_stream) != 0))
      return REDIST_ERR_HIP;
    user_src.ext = dev_tables;
    user_dst.ext = dev_tables + nd;
  }
  // intermediate k lives in workspace region k % 2; with few devices its table is rebuilt per step,
  // with many the two regions' tables are written once (the shard stride of a region is the largest
  // of its intermediates, so one table per region serves every step)
  int64_t region_stride[2] = {0, 0};
  for (size_t k = 0; k + 1 < n_ops; ++k) region_stride[k & 1] = std::max(region_stride[k & 1], p->shard_stride[k]);
  auto ws_table = [&](size_t k) {
    PtrTable t{};
    if (big) {
      t.ext = dev_tables + (size_t)(2 + (k & 1)) * nd;
      return t;
    }
    char* base = static_cast<char*>(workspace) + p->region_off[k];
    for (int d = 0; d < nd; ++d) t.p[d] = base + (int64_t)d * p->shard_stride[k];
    return t;
  };
  if (big) {
    for (size_t k = 0; k + 1 < n_ops && k < 2; ++k) {
      char* base = static_cast<char*>(workspace) + p->region_off[k];
      if (launch_ptr_table_strided(base, region_stride[k], nd, dev_tables + (size_t)(2 + k) * nd, hip_stream) != 0)
        return REDIST_ERR_HIP;
    }
  }
  for (size_t k = op_begin; k < op_end; ++k) {
    PtrTable s = k == 0 ? user_src : ws_table(k - 1);
    PtrTable d = k + 1 == n_ops ? user_dst : ws_table(k);
    const CopyOp& op = p->ops[k];
    int e = op.cell.enabled
                ? launch_cell_op(op.kind, op.cell, desc + p->cbox_off[k], desc + p->clist_off[k], s, d, hip_stream)
                : op.row.enabled
                ? launch_row_op(op.kind, op.row, desc + p->rbox_off[k], desc + p->rpiece_off[k], desc + p->rlist_off[k], s,
                                d, hip_stream)
                : launch_copy_op(op, desc + p->boxes_off[k], desc + p->list_off[k], s, d, hip_stream);
    if (e != 0) return REDIST_ERR_HIP;
  }
  return REDIST_OK;
}

static redist_status execute_impl(redist_plan* p, const void* const* src_shards, void* const* dst_shards,
                                  void* workspace, void* hip_stream, int64_t op_begin, int64_t op_end) {
  if (!p) return REDIST_ERR_NULL;
  if (op_begin < 0 || op_end > (int64_t)p->ops.size() || op_begin >= op_end) return REDIST_ERR_BAD_ARG;
  if (!p->prepared) {
    redist_status s = plan_prepare_impl(p);
    if (s != REDIST_OK) return s;
  }
  {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return REDIST_ERR_HIP;
    if (dev != p->device) return REDIST_ERR_UNSUPPORTED;  // descriptors live on the device the plan was prepared on
  }
  return enqueue_ops(p, p->dev_blob, src_shards, dst_shards, workspace, hip_stream, (size_t)op_begin, (size_t)op_end);
}

redist_status redist_execute(redist_plan* p, const void* const* src_shards, void* const* dst_shards, void* workspace,
                             void* hip_stream) {
  try {
    if (!p || !src_shards || !dst_shards) return REDIST_ERR_NULL;
    return execute_impl(p, src_shards, dst_shards, workspace, hip_stream, 0, (int64_t)p->ops.size());
  } catch (...) {
    return REDIST_ERR_INTERNAL;
  }
}

redist_status redist_execute_range(redist_plan* p, const void* const* src_shards, void* const* dst_shards, void* workspace,
                                   void* hip_stream, int32_t op_begin, int32_t op_end) {
  try {
    return execute_impl(p, src_shards, dst_shards, workspace, hip_stream, op_begin, op_end);
  } catch (...) {
    return REDIST_ERR_INTERNAL;
  }
}

// ---- the entry point that allocates nothing ----
int32_t redist_plan_static_fits(const redist_plan* p) {
  if (!p) return -1;
  return p->core.ndev <= kMaxExecDevices && (int64_t)p->blob.size() <= (int64_t)REDIST_STATIC_DESC_BYTES &&
                 p->workspace_bytes <= (int64_t)REDIST_STATIC_SCRATCH_BYTES - (int64_t)REDIST_STATIC_DESC_BYTES
             ? 1 : 0;
}

redist_status redist_execute_static(redist_plan* p, const void* const* src_shards, void* const* dst_shards,
                                    void* hip_stream) {
  try {
    if (!p || !src_shards || !dst_shards) return REDIST_ERR_NULL;
    if (redist_plan_static_fits(p) != 1) return REDIST_ERR_UNSUPPORTED;
    static_assert(kStaticScratchBytes == REDIST_STATIC_SCRATCH_BYTES, "header and kernels must agree on the scratch size");
    char* scratch = nullptr;
    if (static_scratch_base(reinterpret_cast<void**>(&scratch)) != 0 || !scratch) return REDIST_ERR_HIP;
    // layout of the area: [descriptors, REDIST_STATIC_DESC_BYTES | intermediates of a multi-launch plan].
    // The descriptors travel on every call: a graph that recorded this call replays the upload with it, whoever
    // used the area in between.
    if (launch_upload(p->blob.data(), p->blob.size(), scratch, hip_stream) != 0) return REDIST_ERR_HIP;
    return enqueue_ops(p, scratch, src_shards, dst_shards, scratch + REDIST_STATIC_DESC_BYTES, hip_stream, 0,
                       p->ops.size());
  } catch (...) {
    return REDIST_ERR_INTERNAL;
  }
}

redist_status redist_copy_baseline(void* dst, const void* src, int64_t bytes, void* hip_stream) {
  if (!dst || !src) return REDIST_ERR_NULL;
  if (bytes < 0 || (bytes & 15) || (reinterpret_cast<uintptr_t>(dst) & 15u) || (reinterpret_cast<uintptr_t>(src) & 15u))
    return REDIST_ERR_BAD_ARG;
  return launch_copy_baseline(dst, src, bytes, hip_stream) == 0 ? REDIST_OK : REDIST_ERR_HIP;
}

const char* redist_status_string(redist_status s) {
  switch (s) {
    case REDIST_OK: return "ok";
    case REDIST_ERR_NULL: return "null pointer";
    case REDIST_ERR_BAD_MESH: return "bad mesh";
    case REDIST_ERR_ILL_FORMED: return "ill-formed distributed type";
    case REDIST_ERR_GLOBAL_MISMATCH: return "source and target global types differ";
    case REDIST_ERR_BAD_ELEM_SIZE: return "element size must be 1, 2, 4, 8 or 16";
    case REDIST_ERR_WORKSPACE: return "workspace required";
    case REDIST_ERR_HIP: return "HIP error";
    case REDIST_ERR_INTERNAL: return "internal planner error";
    case REDIST_ERR_BAD_ARG: return "bad argument";
    case REDIST_ERR_UNSUPPORTED: return "unsupported by the executor (or beyond the limits of the entry point called)";
    case REDIST_ERR_SEARCH_BUDGET: return "planner search budget exhausted";
    default: return "unknown status";
  }
}

}  // extern "C"
