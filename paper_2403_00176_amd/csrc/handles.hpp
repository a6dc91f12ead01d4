// Definitions of the opaque handle types of the C ABI.
#pragma once
#include "internal.hpp"
#include "launch.hpp"

struct sod2_graph_s { sod2::Graph g; };
struct sod2_rdp_s { sod2::Rdp r; };
struct sod2_plan_s { sod2::Plan p; };
struct sod2_binding_s {
  const sod2::Plan* plan = nullptr;
  std::vector<int64_t> symbols;
  sod2::BindResult b;
  std::vector<int> planned_decisions;       // decisions b was planned with
  std::vector<int64_t> planned_exec;        // NonZero counts b was planned with
  std::vector<int64_t> last_exec;           // NonZero counts found by the last run
  std::vector<int> forced;                  // decisions forced on the next runs
  bool has_forced = false;
  int force_variant = -1;
  int force_splits = 0;                     // 0 automatic, 1 never split k, n > 1 that many k ranges where possible
  bool profiling = false;
  const void* constants = nullptr;          // constants derived from the weights (folded LayerNorms), or null: not folded
  size_t constants_bytes = 0;
  std::vector<int> last_decisions;
  sod2::BindResult executed;                // plan of the last run when it contained Switches
  bool has_executed = false;
  std::vector<sod2_launch_record> records;
  std::vector<sod2_trace_entry> trace;      // executed steps of the last run
  std::vector<sod2::Launch> launches;       // one per executed step that runs a kernel
  bool launches_valid = false;
  void* events = nullptr;                   // profiling events, owned by run.hip
  int n_events = 0;
  ~sod2_binding_s();
};
namespace sod2 {
void set_error(const std::string& m);
void destroy_events(void* events, int n);   // run.hip
}
