// Internal data model of the AoT multi-stream DAG executor (not part of the C ABI).
#pragma once

#include <cstdarg>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <string>
#include <vector>

#include "nimble_graph.h"
#include "ng_device.h"

namespace ng {

constexpr unsigned kDefaultSpinLimit = 1u << 22;     // a few seconds of polling
enum Phase { BUILDING = 0, SCHEDULED = 1, PLANNED = 2, BOUND = 3, CAPTURED = 4 };

struct Shape {
    int64_t n = 0, c = 0, h = 0, w = 0;
    int64_t elems() const { return n * c * h * w; }
    bool operator==(const Shape& o) const { return n == o.n && c == o.c && h == o.h && w == o.w; }
};

struct Node {
    int op = 0;
    ng_op_params p{};
    std::vector<int> preds;
    std::vector<const void*> weights;
    Shape out;
    bool is_output = false;
};

// Result of the stream-assignment pass (Algorithm 1 + Appendix A of the paper).
struct Schedule {
    std::vector<std::pair<int, int>> meg;      // E', sorted
    int n_matching = 0;                        // |M| of Step 3
    std::vector<int> chain_of;                 // Steps 4-5
    int n_chains = 0;
    std::vector<int> stream_of;
    int n_streams = 0;
    std::vector<std::pair<int, int>> sync;     // Lambda, sorted
    std::vector<int> event_of;
    int n_events = 0;
    std::vector<int> order;
    std::vector<std::vector<int>> waits;       // per consumer, producers ascending
    std::vector<int> fork, join;
    std::vector<char> solo;                    // node is comparable with every other node (no task can run beside it)
};

// One entry of the task table: everything a launch needs, resolved ahead of time.
struct Task {
    const void* fn = nullptr;                  // host-side handle of the stand-alone kernel
    const char* name = "";
    int kid = 0;                               // kernel id (ng_device.h)
    long ntiles = 0;                           // workgroup-sized shares of the task
    unsigned grid[3] = {1, 1, 1};
    unsigned block[3] = {1, 1, 1};
    unsigned lds_bytes = 0;
    alignas(16) unsigned char args[kLaunchArgBytes];   // the kernel's single by-value argument struct
    unsigned args_bytes = 0;
};

// The settings of the device-resident planner's cost model that decide between plans of similar
// expected length, where the model is least certain. The defaults replay fastest on the cell-style
// workloads; ng_capture also builds the plans of a few other settings and keeps the one that
// replays fastest on the device at hand (an ahead-of-time trial like the choice of the replay mode).
struct PlanKnobs {
    double sync_far_us = 1.0;        // extra cost of a hand-over when producer and consumer sit on different XCDs (measured 1-2 us)
    double spread_penalty_us = 2.0;  // what spreading a task over all XCDs must gain before it is preferred (its readers go the long way too)
    int p4_rounds = 3;               // rounds on the home XCD from which a windowed task takes 4 outputs per thread
    double sync_near_us = 0.7;       // completion counter -> dependent workgroup running, same XCD (measured)
    double publish_us = 1.2;         // stores drained and counter bumped: the workgroup moves on to its next entry
    double far_run_factor = 1.2;     // a tile whose loads and stores all go through the memory side takes longer
    std::vector<double> task_scale;  // per node: measured / modelled tile time of an earlier plan (empty: the model as it is)
};

constexpr int kPlanSettings = 8;
const PlanKnobs& plan_setting(int k);   // the k-th setting ng_capture tries (0 = the default)

// Output of the device-resident planner (ng_resident_plan.cpp).
struct ResidentPlan {
    int n_wg = 0;                              // persistent workgroups (grid size)
    int xcds = 0;                              // XCDs the streams are spread over
    double est_us = 0;                         // makespan the planner's cost model expects
    std::vector<DevTask> tasks;                // [n_nodes]
    std::vector<DevEntry> entries;             // per-workgroup lists, concatenated
    std::vector<int> wg_first;                 // [n_wg + 1]
    std::vector<int> order;                    // tasks in list order: every workgroup's list is a subsequence of it
    std::vector<int> fused_into;               // [n_nodes] convolution whose tiles also produce this task's result (no entries of its own), or -1
    std::vector<char> elided;                  // [n_nodes] concat with nothing to copy (inputs produced in place): no entries either
    std::vector<double> model_run_us;          // [n_nodes] modelled time from a task's last wait to its last store (0: no workgroups of its own)
};

// What modes 0-3 launch and how the multi-stream HIP graph orders it (ng_launch_graph.cpp).
struct LaunchGraph {
    std::vector<int> nodes;                    // tasks with a kernel node of their own, in submission order
    std::vector<std::vector<int>> deps;        // per entry of `nodes`: the launched tasks it depends on
};

// Measurement switches (the ablations quoted in the design notes) exist only in a build with
// -DNG_MEASUREMENT_KNOBS; the product build reads no environment variable at all.
#ifdef NG_MEASUREMENT_KNOBS
inline const char* knob(const char* name) { return getenv(name); }
#else
inline const char* knob(const char*) { return nullptr; }
#endif
// integer switch, range-checked; `fallback` when unset or malformed
inline long knob_int(const char* name, long lo, long hi, long fallback) {
    const char* e = knob(name);
    if (!e || !*e) return fallback;
    char* end = nullptr;
    const long v = strtol(e, &end, 10);
    return (end && *end == 0 && v >= lo && v <= hi) ? v : fallback;
}

struct Runtime;  // HIP-side state, defined in ng_runtime.hip

}  // namespace ng

struct ng_graph {
    ng::Phase phase = ng::BUILDING;
    std::vector<ng::Node> nodes;
    ng::Schedule sched;
    std::vector<size_t> offset, bytes;
    std::vector<int> alias_of;                           // concat node inside whose output this node's output lives, or -1
    size_t arena_bytes = 0;
    std::vector<ng::Task> tasks;                         // one stand-alone kernel per node (inputs: none)
    std::vector<ng::Task> launch_tasks;                  // what modes 0-3 launch: the same, except that a batch-norm / ReLU directly behind
                                                         // a convolution is applied by that convolution's kernel and has no launch of its own
    std::vector<ng::Task> single_tasks;                  // what the single-stream modes launch: the same, with the weight updates of all streams in one launch
    std::vector<int> launch_fused_into;                  // [n_nodes] that convolution (the node itself: a concat with nothing to copy), or -1
    ng::Runtime* rt = nullptr;
    int mode = NG_MODE_AUTO;
    bool trainable = false;                              // some node updates weights: nothing derived from weight values may be kept across replays
    bool launch_fusion = true;                           // modes 0-3: batch-norm / ReLU applied by the convolution's kernel, in-place concats not launched
    int graph_multi_state = 0;                           // capture-time check of the multi-stream graph: 0 not run, 1 reproduced the single-stream result, -1 did not
    int graph_multi_checked = 0;                         // replays of it that were compared
    int assignment = NG_ASSIGN_ALGORITHM1;               // how ng_schedule forms the streams
    bool memory_reuse = false;                           // ng_plan_memory may give a dead tensor's buffer to a later one
    int auto_mode = NG_MODE_GRAPH_MULTI;                 // what NG_MODE_AUTO resolves to (set by ng_capture)
    float auto_trial_us[3] = {0, 0, 0};                  // trial medians of modes 0, 1, 4
    int resident_wg_per_cu = 0;                          // 0 = pick automatically
    int resident_xcds = 0;                               // XCDs the resident kernel spreads over, 0 = all 8
    unsigned resident_spin_limit = ng::kDefaultSpinLimit; // polls before a wait gives up
    int resident_plan_trials = 8;                        // planner settings ng_capture tries (1 = the default setting only)
    int resident_plan_kept = 0;                          // which of them it kept
    bool dry_run = false;                                // task table built for planning only (host, fake addresses)
    bool resident_all_far = false;                       // treat every edge as crossing XCDs (device-scope fences everywhere)
    std::string err;

    int fail(int code, const char* fmt, ...) {
        char buf[512];
        va_list ap;
        va_start(ap, fmt);
        vsnprintf(buf, sizeof buf, fmt, ap);
        va_end(ap);
        err = buf;
        return code;
    }
};

namespace ng {
// ng_schedule.cpp
void compute_schedule(int n, const std::vector<std::pair<int, int>>& edges, Schedule& out, bool exact);
// ng_kernels.hip: fill the launch descriptor of node v (addresses resolved against `arena`;
// `packed` = node v's share of the library-owned constant memory, see packed_floats).
int build_task(ng_graph* g, int v, char* arena, float* packed, Task& t);
size_t packed_floats(const ng_graph* g, int v);
int pack_constants(ng_graph* g, int v, float* packed, void* stream);
const void* resident_kernel_handle(int build);
const void* empty_kernel_handle();
const void* standalone_kernel_handle(int kid, const char** name);
const void* timed_kernel_handle(int kid);
const void* xcd_probe_kernel_handle();
// ng_launch_graph.cpp
void decide_launch_fusion(const ng_graph* g, const std::vector<Task>& tasks, bool fuse, bool one_stream, std::vector<int>& fused_into);
void make_bn_backward_task(const Task& dgrad, const Task& wgrad, Task& t);
bool can_pair(int kid_first, int kid_second);
void make_pair_task(const Task& first, const Task& second, Task& t);
void make_sgd_batch_task(const std::vector<Task>& tasks, const std::vector<int>& members, std::vector<SgdTile>& table,
                         const SgdTile* table_dev, Task& t);
void build_launch_graph(const ng_graph* g, const std::vector<Task>& tasks, const std::vector<int>& fused_into, LaunchGraph& out);
// ng_resident_plan.cpp: xcds = 0 lets the cost model choose among 1, 2, 4, 8.
int plan_resident(const ng_graph* g, int n_wg, int xcds, const PlanKnobs& knobs, ResidentPlan& plan);
bool resident_plan_is_consistent(const ng_graph* g, const ResidentPlan& plan);
// ng_runtime.hip
void destroy_runtime(ng_graph* g);
}  // namespace ng
