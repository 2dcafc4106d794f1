// Host-side planner: distributed types, base-offset maps, weak shortest-path synthesis and
// lowering to device-level collectives (arXiv 2112.01075, Secs. 3-7).  Plain C++, no GPU code.
#pragma once
#include <cstdint>
#include <string>
#include <vector>

namespace redist {

constexpr int kMaxRank = 8;
constexpr int kMaxDevices = 4096;

enum StepKind { kDynSlice = 0, kAllGather = 1, kAllToAll = 2, kAllPermute = 3, kFused = 4 };
enum Mode { kStepwise = 0, kFusedMode = 1, kNaive = 2 };

// Status values mirror redist_status in the public header.
enum Status {
  kOk = 0, kErrNull = 1, kErrBadMesh = 2, kErrIllFormed = 3, kErrGlobalMismatch = 4, kErrBadElemSize = 5,
  kErrWorkspace = 6, kErrHip = 7, kErrInternal = 8, kErrBadArg = 9, kErrUnsupported = 10, kErrSearchBudget = 11
};

struct TypeSpec {
  std::vector<int64_t> gshape;            // s_t
  std::vector<std::vector<int>> axes;     // per dim, mesh axis ids, minor-to-major
};

// One collective of the lowered sequence, described at device level.
struct Step {
  int kind = kFused;
  int dim_i = -1, dim_j = -1;
  int64_t factor = 1;
  std::vector<int64_t> shape_after;       // local tile shape after the step (rank)
  std::vector<int64_t> offs_after;        // ndev*rank: base offset held by each physical device
  std::vector<int32_t> peers;             // see redist_plan_step_peers
};

struct PlanCore {
  int ndev = 0, rank = 0, elem_size = 0, mode = 0;
  std::vector<int64_t> gshape;
  std::vector<int64_t> shape_src, shape_dst;   // localtype(src), localtype(dst)
  std::vector<int64_t> offs_src, offs_dst;     // T[[src]], T[[dst]] per device (ndev*rank)
  std::vector<Step> steps;
  int64_t cost = 0, weak_cost = 0, height = 0, bound = 0;
  // Which limits of the synthesis were reached (the plan is still correct, but a cheaper lowering -- one that needs
  // no allpermute -- may have gone unseen): bit 0 = more optimal paths than the 64 that are kept, bit 1 = the
  // enumeration of optimal paths stopped at its visit limit, bit 2 = the budget of simulated lowerings ran out.
  uint32_t limits_hit = 0;
};

// Validates the problem (well-formedness, equal global types) and synthesises the plan.
// step_latency_elems: added to the weight of every communicating step (allgather, alltoall) in the search; 0 is the
// paper's cost model.  The reported cost is always the paper's.
Status make_plan(const std::vector<int64_t>& mesh_sizes, const TypeSpec& src, const TypeSpec& dst, int elem_size,
                 int mode, int64_t step_latency_elems, PlanCore* out);

int64_t product(const std::vector<int64_t>& v);

}  // namespace redist
