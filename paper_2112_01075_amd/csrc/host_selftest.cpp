// Host-only self-test of the planner, the descriptor builder and the C-ABI's plan objects, meant to be built with
// AddressSanitizer and UndefinedBehaviorSanitizer (paper_2112_01075_amd/build.py --sanitize).  It makes plans for
// seeded random redistribution problems in every mode and with several option sets, reads every getter and table,
// exercises the plan cache and the error paths, and destroys everything.  No kernel runs: the launchers are
// stubs, and no HIP call is reached (plans are never prepared or executed).
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <random>
#include <vector>

#include "../../include/redist.h"
#include "launch.hpp"

namespace redist {   // stubs for what kernels.hip defines
int launch_copy_op(const CopyOp&, const void*, const void*, const PtrTable&, const PtrTable&, void*) { return 1; }
int launch_row_op(int, const RowOp&, const void*, const void*, const void*, const PtrTable&, const PtrTable&, void*) { return 1; }
int launch_cell_op(int, const CellOp&, const void*, const void*, const PtrTable&, const PtrTable&, void*) { return 1; }
int launch_ptr_table(const void* const*, int, void**, void*) { return 1; }
int launch_ptr_table_strided(void*, int64_t, int, void**, void*) { return 1; }
int launch_copy_baseline(void*, const void*, int64_t, void*) { return 1; }
int static_scratch_base(void**) { return 1; }
int launch_upload(const void*, size_t, void*, void*) { return 1; }
const char* kernel_name_of(int) { return "stub"; }
const char* row_kernel_name_of(int) { return "stub_lds"; }
const char* cell_kernel_name_of(int) { return "stub_cell"; }
}  // namespace redist

namespace {

struct Problem {
  std::vector<int64_t> mesh, gshape;
  std::vector<std::vector<int32_t>> axes[2];
};

// Every mesh axis is replicated or tiles one dimension (rejected when the tiling does not divide it).
bool draw_type(std::mt19937& rng, const Problem& p, std::vector<std::vector<int32_t>>* out) {
  const int r = (int)p.gshape.size();
  out->assign((size_t)r, {});
  for (int a = 0; a < (int)p.mesh.size(); ++a) {
    int pick = (int)(rng() % (uint32_t)(r + 1)) - 1;
    if (pick >= 0) (*out)[(size_t)pick].insert((rng() & 1) ? (*out)[(size_t)pick].begin() : (*out)[(size_t)pick].end(), a);
  }
  for (int t = 0; t < r; ++t) {
    int64_t k = 1;
    for (int a : (*out)[(size_t)t]) k *= p.mesh[(size_t)a];
    if (p.gshape[(size_t)t] % k) return false;
  }
  return true;
}

int check_plan(redist_plan* plan) {
  int touched = 0;
  const int nd = redist_plan_num_devices(plan), r = redist_plan_rank(plan), ns = redist_plan_num_steps(plan);
  std::vector<int64_t> offs((size_t)nd * r), shape((size_t)r);
  for (int k = -1; k < ns; ++k) touched += redist_plan_step_offsets(plan, k, offs.data()) == REDIST_OK;
  for (int k = 0; k < ns; ++k) {
    int32_t kind, di, dj;
    int64_t f;
    if (redist_plan_step(plan, k, &kind, &di, &dj, &f, shape.data()) != REDIST_OK) return -1;
    std::vector<int32_t> peers((size_t)nd * (size_t)(f > 0 ? f : 1));
    if (kind != REDIST_STEP_FUSED) touched += redist_plan_step_peers(plan, k, peers.data()) == REDIST_OK;
  }
  for (int k = 0; k < redist_plan_num_ops(plan); ++k) {
    redist_op_info oi;
    redist_row_info ri;
    if (redist_plan_op_info(plan, k, &oi) != REDIST_OK || redist_plan_op_row_info(plan, k, &ri) != REDIST_OK) return -1;
    std::vector<redist_box> boxes((size_t)oi.n_boxes + 1);
    std::vector<int32_t> dl((size_t)oi.n_dst_list + 1);
    touched += redist_plan_op_tables(plan, k, boxes.data(), dl.data()) == REDIST_OK;
    std::vector<redist_row_box> rb((size_t)ri.n_boxes + 1);
    std::vector<redist_piece> pc((size_t)ri.n_pieces_total + 1);
    std::vector<int32_t> dv((size_t)ri.n_dev_list + 1);
    touched += redist_plan_op_row_tables(plan, k, rb.data(), pc.data(), dv.data()) == REDIST_OK;
    redist_cell_info ci;
    if (redist_plan_op_cell_info(plan, k, &ci) != REDIST_OK) return -1;
    std::vector<redist_cell_box> cb((size_t)ci.n_boxes + 1);
    std::vector<int32_t> cl((size_t)ci.n_list + 1);
    touched += redist_plan_op_cell_tables(plan, k, cb.data(), cl.data()) == REDIST_OK;
    int64_t off, stride;
    touched += redist_plan_op_output(plan, k, &off, &stride) == REDIST_OK;
    touched += redist_plan_op_last_step(plan, k) >= -1;
    touched += redist_plan_step_kernel(plan, k)[0] != 0;
  }
  touched += (int)(redist_plan_cost_elems(plan) + redist_plan_weak_cost_elems(plan) + redist_plan_height_elems(plan) +
                   redist_plan_bound_elems(plan) + redist_plan_peak_live_bytes_per_shard(plan) +
                   redist_plan_workspace_bytes(plan) + redist_plan_footprint_bytes_per_shard(plan) +
                   redist_plan_predicted_ns(plan) + redist_plan_static_fits(plan) > 0);
  for (int w = 0; w < 4; ++w) touched += redist_plan_algorithmic_bytes(plan, w) >= 0;
  touched += redist_plan_search_limits_hit(plan) >= 0;
  return touched;
}

}  // namespace

int main(int argc, char** argv) {
  const int n_problems = argc > 1 ? std::atoi(argv[1]) : 400;
  std::mt19937 rng(211201075u);
  const std::vector<std::vector<int64_t>> meshes = {{2, 2}, {2, 3}, {4, 2}, {2, 2, 2}, {6, 4}, {3, 3, 2}, {1, 4}, {8}, {8, 8}, {64, 4}};
  const std::vector<std::vector<int64_t>> shapes = {{12, 12}, {24, 8}, {4, 6, 8}, {48}, {6, 4, 2, 12}, {36, 24}, {96, 40, 90},
                                                    {512, 24}, {16, 32, 64, 16}, {3, 4, 2, 6, 2, 3, 2, 6},
                                                    {8, 4096}, {4, 6, 2048}, {2, 8, 24, 256}};   // (runs long enough for sibling boxes)
  int made = 0, refused = 0, checks = 0;
  for (int n = 0; n < n_problems; ++n) {
    Problem p;
    p.mesh = meshes[rng() % meshes.size()];
    p.gshape = shapes[rng() % shapes.size()];
    if (!draw_type(rng, p, &p.axes[0]) || !draw_type(rng, p, &p.axes[1])) continue;
    redist_mesh mesh{(int32_t)p.mesh.size(), p.mesh.data()};
    std::vector<int32_t> cnt[2], flat[2];
    redist_type ty[2];
    for (int s = 0; s < 2; ++s) {
      for (auto& l : p.axes[s]) { cnt[s].push_back((int32_t)l.size()); flat[s].insert(flat[s].end(), l.begin(), l.end()); }
      flat[s].push_back(0);
      ty[s] = redist_type{(int32_t)p.gshape.size(), p.gshape.data(), cnt[s].data(), flat[s].data()};
    }
    const int elem = 1 << (rng() % 5);
    for (uint32_t mode = 0; mode <= REDIST_MODE_AUTO; ++mode) {
      redist_options o;
      redist_options_init(&o);
      if (rng() & 1) o.cell_form = 2;   // cell-staged descriptors wherever a launch qualifies
      switch (rng() % 4) {              // sibling boxes: off, default, short runs only; staged boxes kept whole
        case 1: o.sibling_sources = 0; break;
        case 2: o.sibling_sources = 4096; break;
        case 3: o.lds_staging = 2; break;
        default: break;
      }
      switch (rng() % 6) {
        case 1: o.merge_runs = 0; break;
        case 2: o.fold_permute = 0; o.dest_major_min_bytes = 0; break;
        case 3: o.lds_staging = 0; o.max_grid = 7; break;
        case 4: o.span_form = 0; o.unroll = 4; o.step_latency_elems = 50; break;
        case 5: o.dest_major = 0; o.step_latency_elems = 1000000; break;
        default: break;
      }
      redist_plan* plan = nullptr;
      const bool cached = (rng() & 3) == 0;
      redist_status st = redist_plan_create_ex(&mesh, &ty[0], &ty[1], elem, mode, &o, cached, &plan);
      if (st != REDIST_OK) { ++refused; continue; }
      ++made;
      const int c = check_plan(plan);
      if (c < 0) { std::fprintf(stderr, "getter failed on problem %d mode %u\n", n, mode); return 1; }
      checks += c;
      if (cached) {   // a second holder of the same cached plan
        redist_plan* again = nullptr;
        if (redist_plan_create_ex(&mesh, &ty[0], &ty[1], elem, mode, &o, 1, &again) != REDIST_OK || again != plan) return 1;
        redist_plan_destroy(again);
      }
      redist_plan_destroy(plan);
    }
    if ((n & 63) == 63) redist_plan_cache_clear();
  }
  // error paths: null arguments, ill-formed types, bad sizes
  {
    int64_t m2[2] = {2, 2}, g[2] = {8, 6};
    int32_t c0[2] = {1, 1}, f_bad[2] = {0, 0}, c1[2] = {0, 0}, f1[1] = {0};
    redist_mesh mesh{2, m2};
    redist_type bad{2, g, c0, f_bad}, ok{2, g, c1, f1};
    redist_plan* plan = nullptr;
    if (redist_plan_create(&mesh, &bad, &ok, 4, 0, &plan) != REDIST_ERR_ILL_FORMED) return 1;
    if (redist_plan_create(nullptr, &ok, &ok, 4, 0, &plan) != REDIST_ERR_NULL) return 1;
    if (redist_plan_create(&mesh, &ok, &ok, 3, 0, &plan) != REDIST_ERR_BAD_ELEM_SIZE) return 1;
    if (redist_plan_create(&mesh, &ok, &ok, 4, 9, &plan) != REDIST_ERR_BAD_ARG) return 1;
    if (redist_plan_num_steps(nullptr) != -1 || redist_plan_static_fits(nullptr) != -1) return 1;
    redist_plan_destroy(nullptr);
  }
  redist_plan_cache_clear();
  std::printf("host self-test ok: %d plans made, %d problems refused, %d getter results checked\n", made, refused, checks);
  return made > 0 ? 0 : 1;
}
