// GPU part of the ahead-of-time pass and the replay path.
//
// Nimble (arXiv 2012.02732), Section 4.1: the network is pre-run once on the assigned
// streams while every submitted GPU task is recorded (stream capture), the record is
// turned into an executable graph, and each later inference is one graph launch - no
// shape checks, no kernel dispatch, no allocator and no argument marshalling at run time
// (the per-task steps listed in Section 2, "GPU Task Scheduling in DL Frameworks").
// Here the library is itself the launcher, so "recording" means: build the task table
// once (ng_bind), then issue it once under hipStreamBeginCapture (ng_capture).
#include <hip/hip_ext.h>
#include <hip/hip_runtime.h>

#include <algorithm>
#include <chrono>
#include <cstdlib>
#include <cstring>

#include "ng_device.h"
#include "ng_internal.h"

namespace ng {

struct Runtime {
    char* arena = nullptr;
    size_t arena_bytes = 0;
    std::vector<hipStream_t> streams;
    std::vector<hipEvent_t> events;        // one per producer in Lambda
    hipEvent_t fork_event = nullptr;
    std::vector<hipEvent_t> join_events;   // indexed by stream (entry 0 unused)
    hipGraph_t graph[2] = {nullptr, nullptr};
    hipGraphExec_t exec[2] = {nullptr, nullptr};
    hipEvent_t t_start = nullptr, t_stop = nullptr;
    float* constants = nullptr;            // library-owned: repacked weights
    SgdTile* sgd_tiles = nullptr;          // library-owned: the shares of the batched weight updates (modes 0-3)
    float empty_chain_us = 0.f;            // per-node time of a chain of empty kernels (measured on demand)
    unsigned long long* stamps = nullptr;  // device memory: the clock readings of a timed kernel, one pair per workgroup
    size_t stamps_wgs = 0;
    // device-resident replay
    DevPlan plan{};
    void* d_records = nullptr;
    void* d_wg_first = nullptr;
    int* h_error = nullptr;                // pinned host memory
    int n_wg = 0, n_entries = 0;
    std::vector<int> entry_task;           // node of every list entry, in record order (for the timeline)
    std::vector<int> fused_into;           // per node: the convolution that also produces its result, or -1
    std::vector<char> elided;              // per node: a concat with nothing to copy
    std::vector<DevTask> kept_tasks;       // per node: kernel id, tile count and argument block of the installed plan (host copy)
    bool xcd_mapping_ok = false;           // workgroups of the resident grid with equal index mod 8 share an XCD (probed)
    int resident_build = BUILD_FULL;       // which build of the resident kernel the DAG's kernels need
    unsigned epoch = 0;
    size_t done_words = 0;
    int xcds = 0;
    double est_us = 0;
    bool counters_dirty = false;
    int device = -1;                       // the device that was current at ng_bind
    // a graph that trains: copies of the weights its update nodes write, taken when ng_capture starts
    std::vector<std::pair<float*, size_t>> trained;   // (caller's buffer, elements)
    float* trained_copy = nullptr;
};

namespace {

#define NG_HIP(call)                                                                        \
    do {                                                                                    \
        hipError_t e_ = (call);                                                             \
        if (e_ != hipSuccess)                                                               \
            return g->fail(NG_EHIP, "%s failed: %s (%s:%d)", #call, hipGetErrorString(e_), __FILE__, __LINE__); \
    } while (0)

int launch(ng_graph* g, const Task& t, hipStream_t s) {
    if (!t.fn) return NG_OK;                                   // input node: nothing to run
    void* args[1] = {const_cast<unsigned char*>(t.args)};
    NG_HIP(hipLaunchKernel(t.fn, dim3(t.grid[0], t.grid[1], t.grid[2]), dim3(t.block[0], t.block[1], t.block[2]),
                           args, t.lds_bytes, s));
    return NG_OK;
}

// Issue the whole task table once, in submission order. multi = true: every task on its
// assigned stream with the planned event records / waits plus fork and join scaffolding;
// multi = false: everything on the origin stream, no events at all.
int issue_all(ng_graph* g, bool multi) {
    Runtime& rt = *g->rt;
    const Schedule& sc = g->sched;
    hipStream_t origin = rt.streams[0];
    if (!multi) {
        for (int v : sc.order)
            if (int rc = launch(g, g->single_tasks[v], origin)) return rc;
        return NG_OK;
    }
    if (!sc.fork.empty()) {
        NG_HIP(hipEventRecord(rt.fork_event, origin));
        for (int s : sc.fork) NG_HIP(hipStreamWaitEvent(rt.streams[s], rt.fork_event, 0));
    }
    for (int v : sc.order) {
        hipStream_t s = rt.streams[sc.stream_of[v]];
        for (int u : sc.waits[v]) NG_HIP(hipStreamWaitEvent(s, rt.events[sc.event_of[u]], 0));
        if (int rc = launch(g, g->launch_tasks[v], s)) return rc;
        if (sc.event_of[v] >= 0) NG_HIP(hipEventRecord(rt.events[sc.event_of[v]], s));
    }
    for (int s : sc.join) {
        NG_HIP(hipEventRecord(rt.join_events[s], rt.streams[s]));
        NG_HIP(hipStreamWaitEvent(origin, rt.join_events[s], 0));
    }
    return NG_OK;
}

// Single-stream record: pre-run the task table on the origin stream under stream capture.
int capture_single(ng_graph* g, int slot) {
    Runtime& rt = *g->rt;
    hipStream_t origin = rt.streams[0];
    NG_HIP(hipStreamBeginCapture(origin, hipStreamCaptureModeThreadLocal));
    int rc = issue_all(g, false);
    hipGraph_t graph = nullptr;
    hipError_t e = hipStreamEndCapture(origin, &graph);        // always end the capture, even after a failure
    if (rc) {
        if (graph) (void)hipGraphDestroy(graph);
        return rc;
    }
    if (e != hipSuccess) return g->fail(NG_EHIP, "hipStreamEndCapture failed: %s", hipGetErrorString(e));
    rt.graph[slot] = graph;
    NG_HIP(hipGraphInstantiate(&rt.exec[slot], graph, nullptr, nullptr, 0));
    return NG_OK;
}

// Multi-stream record. The library already knows everything a capture of the pre-run
// would discover, so the graph is written down directly: one kernel node per launch, an
// edge from the previous task of the same stream (FIFO order within a stream) and an
// edge for every planned event wait (Lambda). This is node for node and edge for edge
// the graph that capturing issue_all(multi = true) describes; which nodes and which edges
// is decided by host-only code (build_launch_graph), the same that ng_get_graph_edges reports.
int record_multi(ng_graph* g, int slot) {
    Runtime& rt = *g->rt;
    const int n = (int)g->nodes.size();
    LaunchGraph lg;
    build_launch_graph(g, g->tasks, g->launch_fused_into, lg);
    hipGraph_t graph = nullptr;
    NG_HIP(hipGraphCreate(&graph, 0));
    rt.graph[slot] = graph;
    std::vector<hipGraphNode_t> node_of(n, nullptr);
    for (size_t i = 0; i < lg.nodes.size(); ++i) {
        const int v = lg.nodes[i];
        const Task& t = g->launch_tasks[v];
        if (!t.fn) return g->fail(NG_EINVAL, "multi-stream graph: task %d has no kernel", v);
        std::vector<hipGraphNode_t> deps;
        for (int d : lg.deps[i]) {
            if (!node_of[d]) return g->fail(NG_EINVAL, "multi-stream graph: task %d depends on task %d, which has no node yet", v, d);
            deps.push_back(node_of[d]);
        }
        void* args[1] = {const_cast<unsigned char*>(t.args)};
        hipKernelNodeParams kp{};
        kp.func = const_cast<void*>(t.fn);
        kp.gridDim = dim3(t.grid[0], t.grid[1], t.grid[2]);
        kp.blockDim = dim3(t.block[0], t.block[1], t.block[2]);
        kp.sharedMemBytes = t.lds_bytes;
        kp.kernelParams = args;
        kp.extra = nullptr;
        NG_HIP(hipGraphAddKernelNode(&node_of[v], graph, deps.empty() ? nullptr : deps.data(), deps.size(), &kp));
    }
    if (const char* dot = knob("NG_GRAPH_DOT")) (void)hipGraphDebugDotPrint(graph, dot, 0);   // measurement builds: for inspection
    NG_HIP(hipGraphInstantiate(&rt.exec[slot], graph, nullptr, nullptr, 0));
    return NG_OK;
}

// ---- capture-time check of the multi-stream graph -------------------------------------------
// The multi-stream graph and the single-stream graph launch the same kernels with the same
// arguments, so after any execution that respects the graph's edges every byte of the arena is
// the same. The check replays the multi-stream graph several times on an arena whose tensors
// were overwritten with a NaN pattern and compares the whole arena with what the single-stream
// graph left behind. A graph replay that lets a kernel start before its producer (seen on one
// synthetic DAG with this HIP runtime although every edge was in the graph) shows up as
// a stale or poisoned tensor. It is a probabilistic screen, not a proof: an order violation that
// happens in 4 % of launches is caught by 64 replays with probability 0.93.
__global__ __launch_bounds__(256) void poison_kernel(unsigned* p, size_t words) {
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < words; i += (size_t)gridDim.x * 256) p[i] = 0x7FC0DEADu;
}
__global__ __launch_bounds__(256) void mismatch_kernel(const unsigned* a, const unsigned* b, size_t words, unsigned* count) {
    unsigned mine = 0;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < words; i += (size_t)gridDim.x * 256) mine += a[i] != b[i];
    if (mine) atomicAdd(count, mine);
}

// A replay of a graph that trains changes the caller's weights. ng_capture replays many times (pre-run,
// trials, the check of the multi-stream graph): it keeps a copy of every weight buffer an update node
// writes and puts the values back, so that capture leaves the weights as it found them and the check
// compares replays that start from the same weights.
int save_trained_weights(ng_graph* g) {
    Runtime& rt = *g->rt;
    rt.trained.clear();
    if (rt.trained_copy) (void)hipFree(rt.trained_copy), rt.trained_copy = nullptr;
    size_t total = 0;
    for (const Node& nd : g->nodes)
        if (nd.op == NG_OP_SGD_UPDATE) {
            rt.trained.emplace_back(const_cast<float*>(static_cast<const float*>(nd.weights[0])), (size_t)nd.p.cout);
            total += (size_t)nd.p.cout;
        }
    if (total == 0) return NG_OK;
    NG_HIP(hipMalloc(reinterpret_cast<void**>(&rt.trained_copy), total * sizeof(float)));
    size_t at = 0;
    for (auto& w : rt.trained) {
        NG_HIP(hipMemcpyAsync(rt.trained_copy + at, w.first, w.second * sizeof(float), hipMemcpyDeviceToDevice, rt.streams[0]));
        at += w.second;
    }
    NG_HIP(hipStreamSynchronize(rt.streams[0]));
    return NG_OK;
}
int restore_trained_weights(ng_graph* g) {
    Runtime& rt = *g->rt;
    if (!rt.trained_copy) return NG_OK;
    size_t at = 0;
    for (auto& w : rt.trained) {
        NG_HIP(hipMemcpyAsync(w.first, rt.trained_copy + at, w.second * sizeof(float), hipMemcpyDeviceToDevice, rt.streams[0]));
        at += w.second;
    }
    return NG_OK;
}

int issue_poison(ng_graph* g, hipStream_t s) {
    Runtime& rt = *g->rt;
    // everything except the network inputs (their values are the caller's)
    std::vector<std::pair<size_t, size_t>> keep;
    for (size_t v = 0; v < g->nodes.size(); ++v)
        if (g->nodes[v].op == NG_OP_INPUT) keep.emplace_back(g->offset[v], g->offset[v] + g->bytes[v]);
    std::sort(keep.begin(), keep.end());
    size_t at = 0;
    auto fill = [&](size_t lo, size_t hi) -> int {
        if (hi <= lo) return NG_OK;
        const size_t words = (hi - lo) / 4;
        const unsigned blocks = (unsigned)std::min<size_t>((words + 255) / 256, 4096);
        poison_kernel<<<dim3(blocks), dim3(256), 0, s>>>(reinterpret_cast<unsigned*>(rt.arena + lo), words);
        NG_HIP(hipGetLastError());
        return NG_OK;
    };
    for (auto& k : keep) {
        if (int rc = fill(at, k.first)) return rc;
        at = std::max(at, k.second);
    }
    return fill(at, g->arena_bytes);
}

int verify_graph_multi(ng_graph* g, int replays) {
    Runtime& rt = *g->rt;
    hipStream_t s = rt.streams[0];
    g->graph_multi_state = 0;
    g->graph_multi_checked = 0;
    if (g->arena_bytes < 4) return NG_OK;
    const size_t words = g->arena_bytes / 4;
    unsigned* snap = nullptr;
    unsigned* d_count = nullptr;
    NG_HIP(hipMalloc(reinterpret_cast<void**>(&snap), words * 4));
    int rc = NG_OK;
    unsigned mismatches = 0;
    auto hip_ok = [&](hipError_t e, const char* what) {
        if (e != hipSuccess && rc == NG_OK) rc = g->fail(NG_EHIP, "checking the multi-stream graph: %s: %s", what, hipGetErrorString(e));
        return e == hipSuccess;
    };
    if (hip_ok(hipMalloc(reinterpret_cast<void**>(&d_count), sizeof(unsigned)), "hipMalloc") &&
        hip_ok(hipMemsetAsync(d_count, 0, sizeof(unsigned), s), "hipMemsetAsync") && (rc = restore_trained_weights(g)) == NG_OK &&
        (rc = issue_poison(g, s)) == NG_OK &&
        hip_ok(hipGraphLaunch(rt.exec[1], s), "hipGraphLaunch (single stream)") &&
        hip_ok(hipMemcpyAsync(snap, rt.arena, words * 4, hipMemcpyDeviceToDevice, s), "hipMemcpyAsync") &&
        hip_ok(hipStreamSynchronize(s), "hipStreamSynchronize")) {
        if (replays <= 0) {
            // about 40 ms of replays, 8 to 64 of them
            const auto t0 = std::chrono::steady_clock::now();
            if ((rc = restore_trained_weights(g)) == NG_OK && hip_ok(hipGraphLaunch(rt.exec[0], s), "hipGraphLaunch") &&
                hip_ok(hipStreamSynchronize(s), "hipStreamSynchronize")) {
                const double us = std::chrono::duration<double, std::micro>(std::chrono::steady_clock::now() - t0).count();
                replays = (int)std::min(64.0, std::max(8.0, 40000.0 / std::max(us, 1.0)));
            }
        }
        const unsigned blocks = (unsigned)std::min<size_t>((words + 255) / 256, 4096);
        for (int i = 0; i < replays && rc == NG_OK; ++i) {
            if ((rc = issue_poison(g, s)) != NG_OK || (rc = restore_trained_weights(g)) != NG_OK) break;
            if (!hip_ok(hipGraphLaunch(rt.exec[0], s), "hipGraphLaunch")) break;
            mismatch_kernel<<<dim3(blocks), dim3(256), 0, s>>>(reinterpret_cast<const unsigned*>(rt.arena), snap, words, d_count);
            if (!hip_ok(hipGetLastError(), "compare kernel")) break;
            ++g->graph_multi_checked;
        }
        if (rc == NG_OK && hip_ok(hipMemcpyAsync(&mismatches, d_count, sizeof(unsigned), hipMemcpyDeviceToHost, s), "hipMemcpyAsync"))
            hip_ok(hipStreamSynchronize(s), "hipStreamSynchronize");
    }
    (void)hipStreamSynchronize(s);
    if (d_count) (void)hipFree(d_count);
    (void)hipFree(snap);
    if (rc != NG_OK) return rc;
    g->graph_multi_state = mismatches == 0 && g->graph_multi_checked > 0 ? 1 : -1;
    // leave the arena as a normal replay leaves it
    if (int rc2 = restore_trained_weights(g)) return rc2;
    NG_HIP(hipGraphLaunch(rt.exec[1], s));
    NG_HIP(hipStreamSynchronize(s));
    return NG_OK;
}

int make_plan(ng_graph* g, const PlanKnobs& knobs, ResidentPlan& hp);
int install_plan(ng_graph* g, const ResidentPlan& hp);
int tune_resident(ng_graph* g);

// Device-resident replay: plan on the host (ng_resident_plan.cpp), upload, keep the handles.
int build_resident(ng_graph* g) {
    Runtime& rt = *g->rt;
    const int n = (int)g->nodes.size();
    int dev = 0, cus = 0, per_cu = 0;
    NG_HIP(hipGetDevice(&dev));
    NG_HIP(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
    rt.resident_build = BUILD_LEAN;
    for (const Task& t : g->tasks)
        if (t.fn && is_train_kernel(t.kid)) rt.resident_build = BUILD_TRAIN;
    for (const Task& t : g->tasks)
        if (t.fn && !is_lean_kernel(t.kid) && !is_train_kernel(t.kid)) {
            if (rt.resident_build == BUILD_TRAIN && in_build(BUILD_TRAIN, t.kid)) continue;
            if (rt.resident_build == BUILD_TRAIN) return g->fail(NG_EINVAL, "device-resident replay: kernel %s does not belong in a graph that trains", t.name);
            rt.resident_build = BUILD_FULL;
        }
    NG_HIP(hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, resident_kernel_handle(rt.resident_build), kGroup, 0));
    if (per_cu < 1 || cus < 8) return g->fail(NG_EHIP, "device-resident replay: kernel does not fit (%d per CU, %d CUs)", per_cu, cus);
    per_cu = std::min(per_cu, g->resident_wg_per_cu > 0 ? g->resident_wg_per_cu : 1);   // one per CU: two slow each other's hand-overs down
    const int n_wg = cus * per_cu / 8 * 8;
    // The plan keeps a stream's tensors and completion counters in the L2 of "its" XCD and takes
    // workgroups with the same index mod 8 to share one. Check that on this device with this grid; if
    // it does not hold, every hand-over goes through device scope instead (correct whatever the
    // mapping, only slower).
    {
        int* d_xcd = nullptr;
        NG_HIP(hipMalloc(reinterpret_cast<void**>(&d_xcd), (size_t)n_wg * sizeof(int)));
        void* probe_args[1] = {&d_xcd};
        hipError_t pe = hipLaunchKernel(xcd_probe_kernel_handle(), dim3(n_wg), dim3(kGroup), probe_args, 0, rt.streams[0]);
        std::vector<int> xcd_of((size_t)n_wg, -1);
        if (pe == hipSuccess) pe = hipMemcpyAsync(xcd_of.data(), d_xcd, (size_t)n_wg * sizeof(int), hipMemcpyDeviceToHost, rt.streams[0]);
        if (pe == hipSuccess) pe = hipStreamSynchronize(rt.streams[0]);
        (void)hipFree(d_xcd);
        if (pe != hipSuccess) return g->fail(NG_EHIP, "device-resident replay: XCD probe: %s", hipGetErrorString(pe));
        // the dispatcher deals workgroups out round-robin, starting at an XCD that depends on what ran
        // before: which XCD a class gets does not matter, only that a class stays together
        rt.xcd_mapping_ok = true;
        for (int w = 0; w < n_wg; ++w) rt.xcd_mapping_ok = rt.xcd_mapping_ok && xcd_of[w] >= 0 && xcd_of[w] == xcd_of[w % 8];
        if (!rt.xcd_mapping_ok && knob("NG_PLAN_DEBUG")) {
            fprintf(stderr, "XCD probe mismatch:");
            for (int w = 0; w < std::min(n_wg, 48); ++w) fprintf(stderr, " %d", xcd_of[w]);
            fprintf(stderr, "\n");
        }
        if (!rt.xcd_mapping_ok) g->resident_all_far = true;
    }
    unsigned* d_done = nullptr;
    int* d_error = nullptr;
    rt.plan.done_stride = (int)knob_int("NG_DONE_STRIDE", 1, 1024, 64);    // one counter per 256 bytes
    rt.plan.poll_sleep = (int)knob_int("NG_POLL_SLEEP", 0, 2, 1);
    rt.done_words = (size_t)n * rt.plan.done_stride;
    NG_HIP(hipMalloc(&d_done, (10 * rt.done_words + 18) * sizeof(unsigned)));  // device-scope counters, the XCD-local ones, 8 per-XCD first-level ones, 8 class records
    NG_HIP(hipMalloc(&d_error, sizeof(int)));
    NG_HIP(hipHostMalloc(reinterpret_cast<void**>(&rt.h_error), sizeof(int), hipHostMallocDefault));
    *rt.h_error = 0;
    NG_HIP(hipMemset(d_done, 0, (10 * rt.done_words + 18) * sizeof(unsigned)));
    NG_HIP(hipMemset(d_error, 0, sizeof(int)));
    rt.plan.done = d_done;
    rt.plan.done_near = d_done + rt.done_words;
    rt.plan.done_xcd = d_done + 2 * rt.done_words;
    rt.plan.xcc_seen = rt.xcd_mapping_ok && !g->resident_all_far
                           ? reinterpret_cast<unsigned long long*>(d_done + ((10 * rt.done_words + 1) & ~(size_t)1))   // 8-byte aligned, behind the counters
                           : nullptr;
    rt.plan.error_dev = d_error;
    rt.plan.error_host = rt.h_error;
    rt.plan.spin_limit = g->resident_spin_limit;
    rt.n_wg = n_wg;
    rt.epoch = 0;
    rt.counters_dirty = false;
    ResidentPlan hp;
    if (int rc = make_plan(g, PlanKnobs(), hp)) return rc;
    return install_plan(g, hp);
}

// The planner's output for one setting of its cost model, self-checked.
int make_plan(ng_graph* g, const PlanKnobs& knobs_in, ResidentPlan& hp) {
    PlanKnobs knobs = knobs_in;
    if (const char* e = knob("NG_KNOBS")) {                   // measurement builds only: "far,spread,p4,near,publish,farrun"
        PlanKnobs k = knobs;
        const bool parsed = sscanf(e, "%lf,%lf,%d,%lf,%lf,%lf", &k.sync_far_us, &k.spread_penalty_us, &k.p4_rounds, &k.sync_near_us, &k.publish_us, &k.far_run_factor) == 6;
        auto sane = [](double v) { return v >= 0.0 && v <= 100.0; };
        if (parsed && sane(k.sync_far_us) && sane(k.spread_penalty_us) && k.p4_rounds >= 1 && sane(k.sync_near_us) && sane(k.publish_us) &&
            k.far_run_factor >= 0.5 && k.far_run_factor <= 10.0)
            knobs = k;
    }
    if (plan_resident(g, g->rt->n_wg, g->resident_xcds, knobs, hp) != NG_OK)
        return g->fail(NG_EINVAL, "device-resident replay: a node has more than %d E' parents", NG_MAX_PREDS);
    // never launch a plan that does not pass its own check (coverage, one common order with parents first, counts):
    // a wait that can never be satisfied would only end at the spin limit
    if (!resident_plan_is_consistent(g, hp)) return g->fail(NG_EINVAL, "device-resident replay: the plan failed its self-check");
    return NG_OK;
}

// Upload a plan: one record per list entry and the list heads. Replaces the plan that was there
// (the caller has waited for its last replay). A task's counter grows per replay by the number
// of workgroups the plan gave it, so the counters of another plan mean nothing to this one: the
// next launch starts from zeroed counters and epoch 1 again.
int install_plan(ng_graph* g, const ResidentPlan& hp) {
    Runtime& rt = *g->rt;
    const int n_wg = rt.n_wg;
    const std::vector<DevTask>& tasks = hp.tasks;
    const std::vector<DevEntry>& entries = hp.entries;
    const std::vector<int>& wg_first = hp.wg_first;
    if (rt.d_records) (void)hipFree(rt.d_records), rt.d_records = nullptr;
    if (rt.d_wg_first) (void)hipFree(rt.d_wg_first), rt.d_wg_first = nullptr;
    if (rt.plan.trace) (void)hipFree(rt.plan.trace), rt.plan.trace = nullptr;   // sized for the old lists: tracing is off again
    rt.xcds = hp.xcds;
    rt.est_us = hp.est_us;
    // one self-contained record per entry: the kernel never touches the task table itself
    std::vector<DevRecord> records(std::max<size_t>(entries.size(), 1));
    std::memset(records.data(), 0, records.size() * sizeof(DevRecord));
    rt.entry_task.assign(entries.size(), 0);
    rt.fused_into = hp.fused_into;
    rt.elided = hp.elided;
    rt.kept_tasks = hp.tasks;
    for (size_t e = 0; e < entries.size(); ++e) {
        rt.entry_task[e] = entries[e].task;
        const DevTask& t = tasks[entries[e].task];
        DevRecord& r = records[e];
        r.task = entries[e].task, r.kid = t.kid, r.ntiles = t.ntiles, r.n_parents = t.n_parents;
        r.tile_begin = entries[e].tile_begin, r.tile_step = entries[e].tile_step;
        r.flags = (t.far_in != 0 ? 1 : 0) | (t.release_far != 0 ? 2 : 0) | ((t.publish & 1u) ? 4 : 0) | ((t.publish & 2u) ? 8 : 0) | ((t.publish & 4u) ? 16 : 0) | ((int)t.n_late << 8);
        r.subs = entries[e].subs | (entries[e].xcd_peers << 8);
        for (int j = 0; j < NG_MAX_PREDS; ++j) r.parent[j] = t.parent[j] | (((t.parent_far >> j) & 1u) ? (int)0x80000000u : 0);
        std::memcpy(r.need, t.need, sizeof r.need);
        std::memcpy(r.args, t.args, sizeof r.args);
    }

    NG_HIP(hipMalloc(&rt.d_records, records.size() * sizeof(DevRecord)));
    NG_HIP(hipMalloc(&rt.d_wg_first, wg_first.size() * sizeof(int)));
    NG_HIP(hipMemcpy(rt.d_records, records.data(), records.size() * sizeof(DevRecord), hipMemcpyHostToDevice));
    NG_HIP(hipMemcpy(rt.d_wg_first, wg_first.data(), wg_first.size() * sizeof(int), hipMemcpyHostToDevice));
    rt.plan.records = static_cast<const DevRecord*>(rt.d_records);
    rt.plan.wg_first = static_cast<const int*>(rt.d_wg_first);
    rt.n_entries = wg_first[n_wg];
    if (rt.epoch != 0) rt.counters_dirty = true;
    return NG_OK;
}

int launch_resident(ng_graph* g);
void pick_auto_mode(ng_graph* g);

// The planner's cost model cannot tell plans of similar expected length apart (its figures are a
// few tenths of a microsecond off per task, and which of them matter depends on the DAG). So a
// few settings of the knobs it is least sure about are planned, each distinct plan is replayed
// a few times, and the fastest one stays - measured ahead of time on the device at hand, like
// everything else that is fixed before the first real replay.
int tune_resident(ng_graph* g) {
    const int trials = std::min(g->resident_plan_trials, kPlanSettings);
    g->resident_plan_kept = 0;
    if (trials <= 1 || knob("NG_NO_TUNE")) return NG_OK;
    const int saved_mode = g->mode;
    g->mode = NG_MODE_DEVICE_RESIDENT;
    auto time_installed = [&](float* median_us) -> int {
        std::vector<float> us;
        int reps = 3 + 11;
        for (int rep = 0; rep < reps; ++rep) {
            const auto t0 = std::chrono::steady_clock::now();
            int rc = launch_resident(g);
            if (rc == NG_OK) rc = ng_sync(g);
            if (rc != NG_OK) return rc;
            const float t = std::chrono::duration<float, std::micro>(std::chrono::steady_clock::now() - t0).count();
            if (rep >= 3) us.push_back(t);
            if (rep == 2 && t > 3000.f) reps = 3 + 3;             // a long replay: fewer looks
        }
        std::sort(us.begin(), us.end());
        *median_us = us[us.size() / 2];
        return NG_OK;
    };
    std::vector<ResidentPlan> plans;
    std::vector<int> setting_of;
    int best = -1, installed = -1, rc = NG_OK;
    float best_us = 0;
    for (int k = 0; k < trials && rc == NG_OK; ++k) {
        ResidentPlan hp;
        if ((rc = make_plan(g, plan_setting(k), hp)) != NG_OK) break;
        bool seen = false;
        for (const ResidentPlan& q : plans)
            seen = seen || (q.wg_first == hp.wg_first && q.entries.size() == hp.entries.size() &&
                            std::memcmp(q.entries.data(), hp.entries.data(), hp.entries.size() * sizeof(DevEntry)) == 0 &&
                            std::memcmp(q.tasks.data(), hp.tasks.data(), hp.tasks.size() * sizeof(DevTask)) == 0);
        if (seen) continue;
        if ((rc = install_plan(g, hp)) != NG_OK) break;
        installed = (int)plans.size();
        plans.push_back(std::move(hp));
        setting_of.push_back(k);
        float us = 0;
        if ((rc = time_installed(&us)) != NG_OK) break;
        if (knob("NG_PLAN_DEBUG")) fprintf(stderr, "PLAN trial %d: expected %.1f us, replays in %.1f us\n", k, plans.back().est_us, us);
        if (best < 0 || us < best_us) best = installed, best_us = us;
    }
    if (rc == NG_OK && best >= 0 && best != installed) rc = install_plan(g, plans[best]), installed = best;
    if (rc == NG_OK && best >= 0) g->resident_plan_kept = setting_of[best];
    // One more candidate: the kept setting planned again with every task's round time corrected by what
    // a traced replay of the kept plan measured for it (the model's per-kernel figures are averages; a
    // task's own shape can be 30 % off them).
    if (rc == NG_OK && best >= 0 && trials >= kPlanSettings && !knob("NG_NO_MEASURED_PLAN")) {
        const size_t n = g->nodes.size();
        std::vector<double> measured(n, 0.0);
        std::vector<unsigned long long> ticks(4 * n);
        for (int rep = 0; rep < 3 && rc == NG_OK; ++rep) {
            if ((rc = ng_resident_trace(g, 1, nullptr)) != NG_OK) break;
            if ((rc = launch_resident(g)) != NG_OK || (rc = ng_sync(g)) != NG_OK) break;
            if ((rc = ng_resident_trace(g, 0, ticks.data())) != NG_OK) break;
            for (size_t v = 0; v < n; ++v) {
                if (plans[best].model_run_us[v] <= 0 || ticks[4 * v + 3] <= ticks[4 * v + 1]) continue;
                const double us = 0.01 * (double)(ticks[4 * v + 3] - ticks[4 * v + 1]);     // 100 MHz clock
                measured[v] = rep == 0 || measured[v] == 0 ? us : std::min(measured[v], us);
            }
        }
        if (rc == NG_OK) {
            PlanKnobs knobs = plan_setting(setting_of[best]);
            knobs.task_scale.assign(n, 1.0);
            for (size_t v = 0; v < n; ++v) {
                const DevTask& t = plans[best].tasks[v];
                if (measured[v] <= 0 || t.n_late > 0) continue;                 // (a late wait is not tile time)
                knobs.task_scale[v] = std::min(2.5, std::max(0.6, measured[v] / plans[best].model_run_us[v]));
            }
            ResidentPlan hp;
            float us = 0;
            if ((rc = make_plan(g, knobs, hp)) == NG_OK && (rc = install_plan(g, hp)) == NG_OK && (rc = time_installed(&us)) == NG_OK) {
                if (knob("NG_PLAN_DEBUG")) fprintf(stderr, "PLAN trial with measured task times: expected %.1f us, replays in %.1f us\n", hp.est_us, us);
                if (us < best_us) g->resident_plan_kept = kPlanSettings;
                else rc = install_plan(g, plans[best]);
            }
        }
    }
    g->mode = saved_mode;
    return rc;
}

int launch_resident(ng_graph* g) {
    Runtime& rt = *g->rt;
    if (!rt.d_records) return g->fail(NG_ESTATE, "device-resident replay was not prepared");
    hipStream_t origin = rt.streams[0];
    if (rt.counters_dirty) {                                   // a timed-out replay left partial counts behind
        NG_HIP(hipStreamSynchronize(origin));
        NG_HIP(hipMemsetAsync(rt.plan.done, 0, (10 * rt.done_words + 18) * sizeof(unsigned), origin));   // on the stream of the launch below
        NG_HIP(hipMemsetAsync(rt.plan.error_dev, 0, sizeof(int), origin));
        *rt.h_error = 0;
        rt.epoch = 0;
        rt.counters_dirty = false;
    }
    rt.plan.spin_limit = g->resident_spin_limit;
    unsigned epoch = ++rt.epoch;
    void* args[2] = {&rt.plan, &epoch};
    NG_HIP(hipLaunchKernel(resident_kernel_handle(rt.resident_build), dim3(rt.n_wg), dim3(kGroup), args, 0, origin));
    return NG_OK;
}

// NG_MODE_AUTO = the fastest of the candidates that were tried (a trial time of 0 means: not a candidate)
void pick_auto_mode(ng_graph* g) {
    const int candidates[3] = {NG_MODE_GRAPH_MULTI, NG_MODE_GRAPH_SINGLE, NG_MODE_DEVICE_RESIDENT};
    g->auto_mode = NG_MODE_GRAPH_SINGLE;
    float best = 0.f;
    for (int i = 0; i < 3; ++i) {
        if (g->auto_trial_us[i] <= 0.f || (i == 0 && g->graph_multi_state != 1)) continue;
        if (best <= 0.f || g->auto_trial_us[i] < best) best = g->auto_trial_us[i], g->auto_mode = candidates[i];
    }
}

}  // namespace

void destroy_runtime(ng_graph* g) {
    Runtime* rt = g->rt;
    if (!rt) return;
    for (int i = 0; i < 2; ++i) {
        if (rt->exec[i]) (void)hipGraphExecDestroy(rt->exec[i]);
        if (rt->graph[i]) (void)hipGraphDestroy(rt->graph[i]);
    }
    for (hipEvent_t e : rt->events) (void)hipEventDestroy(e);
    for (hipEvent_t e : rt->join_events)
        if (e) (void)hipEventDestroy(e);
    if (rt->fork_event) (void)hipEventDestroy(rt->fork_event);
    if (rt->t_start) (void)hipEventDestroy(rt->t_start);
    if (rt->t_stop) (void)hipEventDestroy(rt->t_stop);
    if (rt->constants) (void)hipFree(rt->constants);
    if (rt->sgd_tiles) (void)hipFree(rt->sgd_tiles);
    if (rt->d_records) (void)hipFree(rt->d_records);
    if (rt->d_wg_first) (void)hipFree(rt->d_wg_first);
    if (rt->plan.done) (void)hipFree(rt->plan.done);
    if (rt->plan.error_dev) (void)hipFree(rt->plan.error_dev);
    if (rt->plan.trace) (void)hipFree(rt->plan.trace);
    if (rt->h_error) (void)hipHostFree(rt->h_error);
    if (rt->stamps) (void)hipFree(rt->stamps);
    if (rt->trained_copy) (void)hipFree(rt->trained_copy);
    delete rt;
    g->rt = nullptr;
}

}  // namespace ng

using namespace ng;

extern "C" {

int ng_bind(ng_graph* g, void* arena, size_t arena_bytes, void* const* hip_streams, int n_streams) {
    if (!g) return NG_EINVAL;
    if (g->phase < PLANNED) return g->fail(NG_ESTATE, "ng_bind: call ng_plan_memory first");
    if (!arena || !hip_streams) return g->fail(NG_EINVAL, "ng_bind: null arena or stream array");
    if ((reinterpret_cast<uintptr_t>(arena) & 255) != 0) return g->fail(NG_EINVAL, "ng_bind: arena must be 256-byte aligned");
    if (arena_bytes < g->arena_bytes)
        return g->fail(NG_ENOMEM, "ng_bind: arena has %zu bytes, the plan needs %zu", arena_bytes, g->arena_bytes);
    if (n_streams < g->sched.n_streams)
        return g->fail(NG_ENOMEM, "ng_bind: %d streams given, the schedule uses %d", n_streams, g->sched.n_streams);
    for (int a = 0; a < g->sched.n_streams; ++a)
        for (int b = a + 1; b < g->sched.n_streams; ++b)
            if (hip_streams[a] == hip_streams[b])
                return g->fail(NG_EINVAL, "ng_bind: streams %d and %d are the same handle; the schedule needs distinct streams", a, b);
    hipPointerAttribute_t attr;
    if (hipPointerGetAttributes(&attr, arena) != hipSuccess || attr.type != hipMemoryTypeDevice) {
        (void)hipGetLastError();
        return g->fail(NG_EINVAL, "ng_bind: arena is not device memory");
    }
    destroy_runtime(g);
    g->rt = new Runtime();
    Runtime& rt = *g->rt;
    rt.arena = static_cast<char*>(arena);
    rt.arena_bytes = arena_bytes;
    NG_HIP(hipGetDevice(&rt.device));
    for (int s = 0; s < g->sched.n_streams; ++s) rt.streams.push_back(static_cast<hipStream_t>(hip_streams[s]));

    // constant memory: weights repacked once, ahead of time, into the order the kernels read them
    std::vector<size_t> const_off(g->nodes.size() + 1, 0);
    for (size_t v = 0; v < g->nodes.size(); ++v) const_off[v + 1] = const_off[v] + ((packed_floats(g, (int)v) + 63) & ~(size_t)63);
    if (const_off.back() > 0) {
        NG_HIP(hipMalloc(reinterpret_cast<void**>(&rt.constants), const_off.back() * sizeof(float)));
        for (int v = 0; v < (int)g->nodes.size(); ++v)
            if (int rc = pack_constants(g, v, rt.constants + const_off[v], rt.streams[0])) return rc;
        NG_HIP(hipStreamSynchronize(rt.streams[0]));
    }
    g->tasks.assign(g->nodes.size(), Task());
    for (int v = 0; v < (int)g->nodes.size(); ++v)
        if (int rc = build_task(g, v, rt.arena, rt.constants ? rt.constants + const_off[v] : nullptr, g->tasks[v])) return rc;
    // Modes 0-3 run one kernel per task, with two exceptions (decide_launch_fusion): a batch-norm / ReLU
    // whose only input is a convolution result is applied by the convolution's kernel while the sums are
    // in registers (the same arithmetic on the same values; both tensors are stored), and a concat all of
    // whose inputs the memory plan placed inside its result is not launched. Such a task has no launch of
    // its own and whatever waits for it waits for what it waited for.
    // Weight updates are gathered into one launch per stream, in the single-stream modes into one launch.
    std::vector<int> single_fused_into;
    decide_launch_fusion(g, g->tasks, g->launch_fusion, false, g->launch_fused_into);
    decide_launch_fusion(g, g->tasks, g->launch_fusion, true, single_fused_into);
    size_t sgd_shares = 0;
    for (int v = 0; v < (int)g->nodes.size(); ++v)
        if (g->tasks[v].kid == KID_SGD && g->tasks[v].fn) sgd_shares += 2 * (size_t)(1 + g->nodes[v].p.cout / kSgdTileElems);   // once per table, rounded up
    if (sgd_shares > 0) NG_HIP(hipMalloc(reinterpret_cast<void**>(&rt.sgd_tiles), sgd_shares * sizeof(SgdTile)));
    std::vector<SgdTile> sgd_table;
    auto fuse_launches = [&](const std::vector<int>& fused_into, std::vector<Task>& out) {
        out = g->tasks;
        std::vector<std::vector<int>> batch(g->nodes.size());       // per last update: the updates its launch carries out, in submission order
        for (int v : g->sched.order) {
            const int u = fused_into[v];
            if (u < 0) continue;
            if (g->tasks[v].kid == KID_SGD && u != v) {
                batch[u].push_back(v);
            } else if (g->tasks[v].kid == KID_BN_DGRAD && g->tasks[u].kid == KID_BN_WGRAD) {
                make_bn_backward_task(g->tasks[v], g->tasks[u], out[u]);
            } else if (g->tasks[v].kid == KID_BN_WGRAD && g->tasks[u].kid == KID_BN_DGRAD) {
                make_bn_backward_task(g->tasks[u], g->tasks[v], out[u]);
            } else if (can_pair(g->tasks[u].kid, g->tasks[v].kid)) {
                make_pair_task(g->tasks[u], g->tasks[v], out[u]);
            } else if (can_pair(g->tasks[v].kid, g->tasks[u].kid)) {
                make_pair_task(g->tasks[v], g->tasks[u], out[u]);
            } else if (g->tasks[v].kid == KID_BN_RAW && g->tasks[u].kid == KID_PW_PX_FWD) {
                const BnRawArgs* bn = reinterpret_cast<const BnRawArgs*>(g->tasks[v].args);
                GemmArgs* conv = reinterpret_cast<GemmArgs*>(out[u].args);
                conv->bn_gamma = bn->gamma, conv->bn_beta = bn->beta, conv->bn_mean = bn->mean, conv->bn_var = bn->var;
                conv->bn_y = bn->y, conv->bn_eps = bn->eps, conv->bn_relu = bn->relu;
            } else if (u != v) {
                const BnArgs* bn = reinterpret_cast<const BnArgs*>(g->tasks[v].args);
                const Epilogue ep{bn->scale, bn->shift, bn->y, bn->relu};
                if (takes_c3_args(g->tasks[u].kid)) reinterpret_cast<C3Args*>(out[u].args)->ep = ep;
                else reinterpret_cast<PwArgs*>(out[u].args)->ep = ep;
            }
            out[v].fn = nullptr;
        }
        for (int u = 0; u < (int)g->nodes.size(); ++u) {
            if (batch[u].empty()) continue;
            batch[u].push_back(u);
            make_sgd_batch_task(g->tasks, batch[u], sgd_table, rt.sgd_tiles, out[u]);
        }
    };
    fuse_launches(g->launch_fused_into, g->launch_tasks);
    fuse_launches(single_fused_into, g->single_tasks);
    if (sgd_table.size() > sgd_shares) return g->fail(NG_EINVAL, "ng_bind: %zu shares of weight updates, room for %zu", sgd_table.size(), sgd_shares);
    if (!sgd_table.empty()) NG_HIP(hipMemcpy(rt.sgd_tiles, sgd_table.data(), sgd_table.size() * sizeof(SgdTile), hipMemcpyHostToDevice));

    rt.events.resize(g->sched.n_events);
    for (auto& e : rt.events) NG_HIP(hipEventCreateWithFlags(&e, hipEventDisableTiming));
    rt.join_events.assign(g->sched.n_streams, nullptr);
    for (int s : g->sched.join) NG_HIP(hipEventCreateWithFlags(&rt.join_events[s], hipEventDisableTiming));
    NG_HIP(hipEventCreateWithFlags(&rt.fork_event, hipEventDisableTiming));
    NG_HIP(hipEventCreate(&rt.t_start));
    NG_HIP(hipEventCreate(&rt.t_stop));
    g->phase = BOUND;
    return NG_OK;
}

int ng_capture(ng_graph* g) {
    if (!g) return NG_EINVAL;
    if (g->phase < BOUND) return g->fail(NG_ESTATE, "ng_capture: call ng_bind first");
    Runtime& rt = *g->rt;
    for (int i = 0; i < 2; ++i) {
        if (rt.exec[i]) (void)hipGraphExecDestroy(rt.exec[i]), rt.exec[i] = nullptr;
        if (rt.graph[i]) (void)hipGraphDestroy(rt.graph[i]), rt.graph[i] = nullptr;
    }
    if (g->trainable)
        if (int rc = save_trained_weights(g)) return rc;
    if (int rc = record_multi(g, 0)) return rc;
    if (int rc = capture_single(g, 1)) return rc;
    // Under a memory plan with reuse over time an address holds several tensors in the course of one replay, produced
    // and read on different XCDs: no XCD-private L2 may keep a line of it (a dirty line of an earlier tensor could be
    // written back over a later one, a clean one could be read in its place). Every store and load of the
    // device-resident replay then goes through device scope, as in the fallback for an unexpected XCD mapping, and the
    // planner runs no task inside another task's tiles (a fused result may live where the host's own input still is).
    if (g->memory_reuse) g->resident_all_far = true;
    if (!rt.d_records)
        if (int rc = build_resident(g)) return rc;
    // the pre-run itself: execute the recorded schedule once so that every kernel is loaded
    NG_HIP(hipGraphLaunch(rt.exec[1], rt.streams[0]));
    NG_HIP(hipStreamSynchronize(rt.streams[0]));
    g->phase = CAPTURED;
    if (rt.d_records)
        if (int rc = tune_resident(g)) return rc;
    // the multi-stream graph has to reproduce the single-stream result before it may be chosen
    if (int rc = verify_graph_multi(g, 0)) return rc;
    // short trial: which way of replaying this schedule is fastest on this DAG
    {
        const int candidates[3] = {NG_MODE_GRAPH_MULTI, NG_MODE_GRAPH_SINGLE, NG_MODE_DEVICE_RESIDENT};
        const int saved = g->mode;
        for (int i = 0; i < 3; ++i) {
            g->auto_trial_us[i] = 0.f;
            if (i == 0 && g->graph_multi_state != 1) continue;
            g->mode = candidates[i];
            std::vector<float> us;
            for (int rep = 0; rep < 2 + 9; ++rep) {
                const auto t0 = std::chrono::steady_clock::now();
                int rc = ng_replay(g);
                if (rc == NG_OK) rc = ng_sync(g);
                if (rc != NG_OK) {
                    g->mode = saved;
                    return rc;
                }
                if (rep >= 2) us.push_back(std::chrono::duration<float, std::micro>(std::chrono::steady_clock::now() - t0).count());
            }
            std::sort(us.begin(), us.end());
            g->auto_trial_us[i] = us[us.size() / 2];
        }
        g->mode = saved;
        pick_auto_mode(g);
    }
    if (g->trainable) {                                        // the caller's weights as ng_capture found them
        if (int rc = restore_trained_weights(g)) return rc;
        NG_HIP(hipStreamSynchronize(rt.streams[0]));
        if (rt.trained_copy) (void)hipFree(rt.trained_copy), rt.trained_copy = nullptr;
        rt.trained.clear();
    }
    return NG_OK;
}

int ng_auto_mode(const ng_graph* g, int* mode, float* trial_us) {
    if (!g) return NG_EINVAL;
    if (g->phase < CAPTURED) return const_cast<ng_graph*>(g)->fail(NG_ESTATE, "ng_auto_mode: call ng_capture first");
    if (mode) *mode = g->auto_mode;
    if (trial_us)
        for (int i = 0; i < 3; ++i) trial_us[i] = g->auto_trial_us[i];
    return NG_OK;
}

int ng_graph_multi_check(const ng_graph* g, int* state, int* replays_compared) {
    if (!g) return NG_EINVAL;
    if (g->phase < CAPTURED) return const_cast<ng_graph*>(g)->fail(NG_ESTATE, "ng_graph_multi_check: call ng_capture first");
    if (state) *state = g->graph_multi_state;
    if (replays_compared) *replays_compared = g->graph_multi_checked;
    return NG_OK;
}

int ng_graph_multi_recheck(ng_graph* g, int replays) {
    if (!g) return NG_EINVAL;
    if (g->phase < CAPTURED) return g->fail(NG_ESTATE, "ng_graph_multi_recheck: call ng_capture first");
    if (replays < 1 || replays > 100000) return g->fail(NG_EINVAL, "ng_graph_multi_recheck: replays must be 1..100000");
    if (g->graph_multi_state < 0) return NG_OK;               // a mismatch once seen stays
    Runtime& rt = *g->rt;
    NG_HIP(hipStreamSynchronize(rt.streams[0]));
    if (g->trainable)
        if (int rc = save_trained_weights(g)) return rc;
    int rc = verify_graph_multi(g, replays);
    if (g->trainable) {                                        // every compared replay started from the caller's weights, and they are back
        if (rc == NG_OK) rc = restore_trained_weights(g);
        (void)hipStreamSynchronize(rt.streams[0]);
        if (rt.trained_copy) (void)hipFree(rt.trained_copy), rt.trained_copy = nullptr;
        rt.trained.clear();
    }
    if (rc != NG_OK) return rc;
    pick_auto_mode(g);
    return NG_OK;
}

int ng_graph_multi_distrust(ng_graph* g) {
    if (!g) return NG_EINVAL;
    if (g->phase < CAPTURED) return g->fail(NG_ESTATE, "ng_graph_multi_distrust: call ng_capture first");
    g->graph_multi_state = -1;
    pick_auto_mode(g);
    return NG_OK;
}

void* ng_tensor_ptr(const ng_graph* g, int id) {
    if (!g || g->phase < BOUND || id < 0 || id >= (int)g->nodes.size()) return nullptr;
    return g->rt->arena + g->offset[id];
}

int ng_replay_mode(ng_graph* g, int mode) {
    if (!g) return NG_EINVAL;
    if (mode < NG_MODE_GRAPH_MULTI || mode > NG_MODE_AUTO) return g->fail(NG_EINVAL, "ng_replay_mode: unknown mode %d", mode);
    g->mode = mode;
    return NG_OK;
}

int ng_replay(ng_graph* g) {
    if (!g) return NG_EINVAL;
    if (g->phase < CAPTURED) return g->fail(NG_ESTATE, "ng_replay: call ng_capture first");
    Runtime& rt = *g->rt;
    switch (g->mode == NG_MODE_AUTO ? g->auto_mode : g->mode) {
        case NG_MODE_GRAPH_MULTI:
            if (g->graph_multi_state < 0)
                return g->fail(NG_ESTATE, "ng_replay: the multi-stream HIP graph did not reproduce the single-stream result when it was checked "
                                          "(%d replays compared); choose another replay mode", g->graph_multi_checked);
            NG_HIP(hipGraphLaunch(rt.exec[0], rt.streams[0]));
            return NG_OK;
        case NG_MODE_GRAPH_SINGLE: NG_HIP(hipGraphLaunch(rt.exec[1], rt.streams[0])); return NG_OK;
        case NG_MODE_EAGER_SINGLE: return issue_all(g, false);
        case NG_MODE_EAGER_MULTI: return issue_all(g, true);
        default: return launch_resident(g);
    }
}

// ---- device-resident replay that allocates nothing -------------------------------------------
// For callers that cannot allocate (code under HIP graph capture, tight serving loops, harnesses that
// forbid hipMalloc): the completion counters, the per-launch XCD records and the error flag of the
// device-resident replay live in a file-scope device array instead of memory from hipMalloc. Each GPU
// holds its own copy of the array (kept until the process ends); its address on a device is looked up
// once, with that device current, and only that address - never the array's name - is used by host code.
// Every call on a GPU shares that GPU's array, so every call first clears the part it uses (with a fill
// kernel, not a memset node, so the call can be captured) and replays as replay number 1.
// Calls that overlap on one GPU - from one graph or from several - race on the array.
constexpr int kStaticMaxNodes = 1024;                                           // nodes of the largest graph this entry point takes
constexpr size_t kStaticScratchWords = 10 * (size_t)kStaticMaxNodes * 64 + 64;  // counters at the default stride + records + flag: 2.5 MiB
static __device__ __align__(256) unsigned scratch[kStaticScratchWords];
constexpr int kMaxDevices = 64;
static unsigned* scratch_on_device[kMaxDevices];                                 // nullptr: not looked up yet

__global__ __launch_bounds__(256) void zero_words_kernel(unsigned* p, size_t words) {
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < words; i += (size_t)gridDim.x * 256) p[i] = 0u;
}

int ng_replay_static(ng_graph* g) {
    if (!g) return NG_EINVAL;
    if (g->phase < CAPTURED) return g->fail(NG_ESTATE, "ng_replay_static: call ng_capture first");
    Runtime& rt = *g->rt;
    if (!rt.d_records) return g->fail(NG_ESTATE, "ng_replay_static: this graph has no device-resident plan");
    const size_t n = g->nodes.size();
    const size_t done_words = n * (size_t)rt.plan.done_stride;
    const size_t xcc_at = (10 * done_words + 1) & ~(size_t)1, error_at = xcc_at + 16, need = error_at + 2;
    if (n > (size_t)kStaticMaxNodes || need > kStaticScratchWords)
        return g->fail(NG_ENOMEM, "ng_replay_static: the graph has %zu nodes and needs %zu words of counters; the static scratch array "
                                  "takes graphs of up to %d nodes (%zu words)", n, need, kStaticMaxNodes, kStaticScratchWords);
    int dev = -1;
    NG_HIP(hipGetDevice(&dev));
    if (dev != rt.device || dev < 0 || dev >= kMaxDevices)
        return g->fail(NG_EINVAL, "ng_replay_static: device %d is current, the graph was bound on device %d", dev, rt.device);
    if (!scratch_on_device[dev]) {
        void* p = nullptr;
        NG_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        scratch_on_device[dev] = static_cast<unsigned*>(p);
    }
    unsigned* base = scratch_on_device[dev];
    DevPlan plan = rt.plan;
    plan.done = base;
    plan.done_near = base + done_words;
    plan.done_xcd = base + 2 * done_words;
    plan.xcc_seen = rt.plan.xcc_seen ? reinterpret_cast<unsigned long long*>(base + xcc_at) : nullptr;
    plan.error_dev = reinterpret_cast<int*>(base + error_at);
    plan.trace = nullptr;
    plan.spin_limit = g->resident_spin_limit;
    hipStream_t origin = rt.streams[0];
    if (*rt.h_error != 0) *rt.h_error = 0;                     // left by a replay that gave up (calls do not overlap, so it has ended)
    const unsigned blocks = (unsigned)std::min<size_t>((need + 255) / 256, 1024);
    zero_words_kernel<<<dim3(blocks), dim3(256), 0, origin>>>(base, need);
    NG_HIP(hipGetLastError());
    unsigned epoch = 1;
    void* args[2] = {&plan, &epoch};
    NG_HIP(hipLaunchKernel(resident_kernel_handle(rt.resident_build), dim3(rt.n_wg), dim3(kGroup), args, 0, origin));
    return NG_OK;
}

int ng_sync(ng_graph* g) {
    if (!g) return NG_EINVAL;
    if (g->phase < BOUND) return g->fail(NG_ESTATE, "ng_sync: call ng_bind first");
    NG_HIP(hipStreamSynchronize(g->rt->streams[0]));
    if (g->rt->h_error && *g->rt->h_error != 0) {
        const int task = *g->rt->h_error - 1;
        g->rt->counters_dirty = true;
        if (*g->rt->h_error == kErrorXcdMapping)
            return g->fail(NG_EHIP, "device-resident replay: workgroups with equal index mod 8 did not share an XCD in this launch, which the "
                                    "plan's use of XCD-local L2s rests on; outputs may be stale");
        return g->fail(NG_EHIP, "device-resident replay: the wait before task %d ran out of spins; outputs are incomplete", task);
    }
    return NG_OK;
}

int ng_resident_config(ng_graph* g, int workgroups_per_cu, int xcds, unsigned spin_limit, int device_scope_everywhere) {
    if (!g) return NG_EINVAL;
    if (workgroups_per_cu < 0 || workgroups_per_cu > 8) return g->fail(NG_EINVAL, "ng_resident_config: workgroups_per_cu must be 0..8");
    if (xcds < 0 || xcds > 8) return g->fail(NG_EINVAL, "ng_resident_config: xcds must be 0..8");
    if (workgroups_per_cu > 0 || xcds > 0 || (device_scope_everywhere != 0) != g->resident_all_far) {
        if (g->phase >= CAPTURED) return g->fail(NG_ESTATE, "ng_resident_config: the gang layout is fixed at ng_capture");
        if (workgroups_per_cu > 0) g->resident_wg_per_cu = workgroups_per_cu;
        if (xcds > 0) g->resident_xcds = xcds;
        g->resident_all_far = device_scope_everywhere != 0;
    }
    g->resident_spin_limit = spin_limit ? spin_limit : kDefaultSpinLimit;
    return NG_OK;
}

int ng_resident_plan_trials(ng_graph* g, int trials) {
    if (!g) return NG_EINVAL;
    if (trials < 1 || trials > 8) return g->fail(NG_EINVAL, "ng_resident_plan_trials: trials must be 1..8");
    if (g->phase >= CAPTURED) return g->fail(NG_ESTATE, "ng_resident_plan_trials: the plan is fixed at ng_capture");
    g->resident_plan_trials = trials;
    return NG_OK;
}

int ng_resident_plan_kept(const ng_graph* g, int* setting) {
    if (!g) return NG_EINVAL;
    if (g->phase < CAPTURED) return const_cast<ng_graph*>(g)->fail(NG_ESTATE, "ng_resident_plan_kept: call ng_capture first");
    if (setting) *setting = g->resident_plan_kept;
    return NG_OK;
}

int ng_resident_trace(ng_graph* g, int enable, unsigned long long* ticks) {
    if (!g) return NG_EINVAL;
    if (g->phase < CAPTURED || !g->rt->d_records) return g->fail(NG_ESTATE, "ng_resident_trace: call ng_capture first");
    Runtime& rt = *g->rt;
    // the kernel keeps three readings per list entry; a node's figures are the extremes over its entries
    const size_t n = g->nodes.size(), entries = rt.entry_task.size(), bytes = std::max<size_t>(entries, 1) * 3 * sizeof(unsigned long long);
    NG_HIP(hipStreamSynchronize(rt.streams[0]));
    if (ticks) {
        if (!rt.plan.trace) return g->fail(NG_ESTATE, "ng_resident_trace: tracing is off");
        std::vector<unsigned long long> raw(std::max<size_t>(entries, 1) * 3);
        NG_HIP(hipMemcpy(raw.data(), rt.plan.trace, bytes, hipMemcpyDeviceToHost));
        for (size_t v = 0; v < n; ++v) ticks[4 * v] = ticks[4 * v + 2] = ~0ull, ticks[4 * v + 1] = ticks[4 * v + 3] = 0;
        for (size_t e = 0; e < entries; ++e) {
            const unsigned long long* r = &raw[3 * e];
            if (r[2] == 0) continue;                             // entry did not run since tracing was switched on
            const size_t v = (size_t)rt.entry_task[e];
            ticks[4 * v] = std::min(ticks[4 * v], r[0]);
            ticks[4 * v + 1] = std::max(ticks[4 * v + 1], r[1]);
            ticks[4 * v + 2] = std::min(ticks[4 * v + 2], r[2]);
            ticks[4 * v + 3] = std::max(ticks[4 * v + 3], r[2]);
        }
        // a fused task ran inside its convolution's tiles: it takes no time of its own, at the moment the tiles are stored
        // (an in-place concat likewise: it is complete the moment its last input is)
        for (size_t v = 0; v < n && v < rt.fused_into.size(); ++v) {
            if (rt.fused_into[v] >= 0) {
                const unsigned long long* c = &ticks[4 * rt.fused_into[v]];
                ticks[4 * v] = ticks[4 * v + 2] = c[2], ticks[4 * v + 1] = ticks[4 * v + 3] = c[3];
            } else if (rt.elided[v]) {
                unsigned long long last = 0;
                for (int u : g->nodes[v].preds) last = std::max(last, ticks[4 * u + 3]);
                ticks[4 * v] = ticks[4 * v + 1] = ticks[4 * v + 2] = ticks[4 * v + 3] = last;
            }
        }
    }
    if (enable) {
        if (!rt.plan.trace) NG_HIP(hipMalloc(reinterpret_cast<void**>(&rt.plan.trace), bytes));
        NG_HIP(hipMemset(rt.plan.trace, 0, bytes));
    } else if (rt.plan.trace) {
        NG_HIP(hipFree(rt.plan.trace));
        rt.plan.trace = nullptr;
    }
    return NG_OK;
}

int ng_resident_xcd_mapping(const ng_graph* g, int* verified) {
    if (!g) return NG_EINVAL;
    if (g->phase < CAPTURED) return const_cast<ng_graph*>(g)->fail(NG_ESTATE, "ng_resident_xcd_mapping: call ng_capture first");
    if (verified) *verified = g->rt->xcd_mapping_ok ? 1 : 0;
    return NG_OK;
}

int ng_resident_fusion(const ng_graph* g, int* host_of) {
    if (!g || !host_of) return NG_EINVAL;
    if (g->phase < CAPTURED) return const_cast<ng_graph*>(g)->fail(NG_ESTATE, "ng_resident_fusion: call ng_capture first");
    for (size_t v = 0; v < g->nodes.size(); ++v)
        host_of[v] = v >= g->rt->fused_into.size() ? -1 : (g->rt->elided[v] ? -2 : g->rt->fused_into[v]);
    return NG_OK;
}

int ng_resident_sizes(const ng_graph* g, int* n_workgroups, int* n_entries, int* xcds, double* expected_us) {
    if (!g) return NG_EINVAL;
    if (g->phase < CAPTURED) return const_cast<ng_graph*>(g)->fail(NG_ESTATE, "ng_resident_sizes: call ng_capture first");
    if (n_workgroups) *n_workgroups = g->rt->n_wg;
    if (n_entries) *n_entries = g->rt->n_entries;
    if (xcds) *xcds = g->rt->xcds;
    if (expected_us) *expected_us = g->rt->est_us;
    return NG_OK;
}

// Time per node of a graph that is a chain of `reps` copies of one kernel node, launched on
// the origin stream: the device runs the copies back to back, each waiting for the one before.
static int chain_time(ng_graph* g, const void* fn, const unsigned grid[3], const unsigned block[3], unsigned lds,
                      void* arg_block, int reps, float* us_per_node) {
    Runtime& rt = *g->rt;
    hipStream_t s = rt.streams[0];
    hipGraph_t graph = nullptr;
    hipGraphExec_t exec = nullptr;
    NG_HIP(hipGraphCreate(&graph, 0));
    hipGraphNode_t prev = nullptr;
    void* args[1] = {arg_block};
    int rc = NG_OK;
    for (int i = 0; i < reps && rc == NG_OK; ++i) {
        hipKernelNodeParams kp{};
        kp.func = const_cast<void*>(fn);
        kp.gridDim = dim3(grid[0], grid[1], grid[2]);
        kp.blockDim = dim3(block[0], block[1], block[2]);
        kp.sharedMemBytes = lds;
        kp.kernelParams = arg_block ? args : nullptr;
        hipGraphNode_t node = nullptr;
        const hipError_t e = hipGraphAddKernelNode(&node, graph, prev ? &prev : nullptr, prev ? 1 : 0, &kp);
        if (e != hipSuccess) rc = g->fail(NG_EHIP, "hipGraphAddKernelNode failed: %s", hipGetErrorString(e));
        prev = node;
    }
    hipError_t e = hipSuccess;
    if (rc == NG_OK && (e = hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0)) != hipSuccess)
        rc = g->fail(NG_EHIP, "hipGraphInstantiate failed: %s", hipGetErrorString(e));
    float best = 1e30f;
    for (int round = 0; round < 4 && rc == NG_OK; ++round) {      // round 0 warms up; best of the other three
        if ((e = hipEventRecord(rt.t_start, s)) != hipSuccess || (e = hipGraphLaunch(exec, s)) != hipSuccess ||
            (e = hipEventRecord(rt.t_stop, s)) != hipSuccess || (e = hipEventSynchronize(rt.t_stop)) != hipSuccess) {
            rc = g->fail(NG_EHIP, "timing a kernel chain failed: %s", hipGetErrorString(e));
            break;
        }
        float ms = 0.f;
        if ((e = hipEventElapsedTime(&ms, rt.t_start, rt.t_stop)) != hipSuccess) {
            rc = g->fail(NG_EHIP, "hipEventElapsedTime failed: %s", hipGetErrorString(e));
            break;
        }
        if (round > 0) best = std::min(best, ms);
    }
    if (exec) (void)hipGraphExecDestroy(exec);
    if (graph) (void)hipGraphDestroy(graph);
    if (rc == NG_OK) *us_per_node = best * 1000.f / (float)reps;
    return rc;
}

int ng_time_replay(ng_graph* g, int reps, float* avg_us) {
    if (!g) return NG_EINVAL;
    if (g->phase < CAPTURED) return g->fail(NG_ESTATE, "ng_time_replay: call ng_capture first");
    if (reps <= 0 || !avg_us) return g->fail(NG_EINVAL, "ng_time_replay: bad argument");
    Runtime& rt = *g->rt;
    hipStream_t s = rt.streams[0];
    NG_HIP(hipEventRecord(rt.t_start, s));
    for (int i = 0; i < reps; ++i)
        if (int rc = ng_replay(g)) return rc;
    NG_HIP(hipEventRecord(rt.t_stop, s));
    if (int rc = ng_sync(g)) return rc;
    float ms = 0.f;
    NG_HIP(hipEventElapsedTime(&ms, rt.t_start, rt.t_stop));
    *avg_us = ms * 1000.f / (float)reps;
    return NG_OK;
}

int ng_time_chain(ng_graph* g, int id, int reps, float* us_per_node) {
    if (!g) return NG_EINVAL;
    if (g->phase < BOUND) return g->fail(NG_ESTATE, "ng_time_chain: call ng_bind first");
    if (id < -1 || id >= (int)g->nodes.size() || reps <= 0 || reps > 10000 || !us_per_node)
        return g->fail(NG_EINVAL, "ng_time_chain: bad argument");
    *us_per_node = 0.f;
    if (id < 0) {
        const unsigned one[3] = {1, 1, 1}, wave[3] = {64, 1, 1};
        return chain_time(g, empty_kernel_handle(), one, wave, 0, nullptr, reps, us_per_node);
    }
    Task& t = g->tasks[id];
    if (!t.fn) return NG_OK;
    return chain_time(g, t.fn, t.grid, t.block, t.lds_bytes, t.args, reps, us_per_node);
}

int ng_time_task(ng_graph* g, int id, int reps, float* isolated_us) {
    if (!g) return NG_EINVAL;
    if (g->phase < BOUND) return g->fail(NG_ESTATE, "ng_time_task: call ng_bind first");
    if (id < 0 || id >= (int)g->nodes.size() || reps <= 0 || !isolated_us) return g->fail(NG_EINVAL, "ng_time_task: bad argument");
    *isolated_us = 0.f;
    if (!g->tasks[id].fn) return NG_OK;
    Runtime& rt = *g->rt;
    if (rt.empty_chain_us <= 0.f)
        if (int rc = ng_time_chain(g, -1, 200, &rt.empty_chain_us)) return rc;
    float c = 0.f;
    if (int rc = ng_time_chain(g, id, reps, &c)) return rc;
    *isolated_us = std::max(c - rt.empty_chain_us, 0.f);
    return NG_OK;
}

// The task as replay mode `mode` really runs it, as a stand-alone launch: the per-task kernel, or the
// convolution with its fused batch-norm (modes 0-3), or the kernel variant of the device-resident plan
// (partition, outputs per thread, fused batch-norm and add_n). false: the task has no kernel of its own
// in that mode (it runs inside another task's kernel, or has nothing to do).
static bool executed_task(const ng_graph* g, int id, int mode, Task& out, const char** name) {
    if (mode == NG_MODE_AUTO) mode = g->auto_mode;
    if (mode != NG_MODE_DEVICE_RESIDENT) {
        out = (mode == NG_MODE_GRAPH_SINGLE || mode == NG_MODE_EAGER_SINGLE) ? g->single_tasks[id] : g->launch_tasks[id];
        if (name) *name = out.name;
        return out.fn != nullptr;
    }
    const Runtime& rt = *g->rt;
    if ((size_t)id >= rt.kept_tasks.size() || !g->tasks[id].fn || rt.fused_into[id] >= 0 || rt.elided[id]) return false;
    const DevTask& d = rt.kept_tasks[id];
    const char* nm = "";
    const void* fn = standalone_kernel_handle(d.kid, &nm);
    if (!fn || d.ntiles <= 0) return false;
    out = Task();
    out.fn = fn, out.name = nm, out.kid = d.kid, out.ntiles = d.ntiles;
    out.grid[0] = (unsigned)d.ntiles, out.block[0] = kBlock;
    static_assert(sizeof out.args >= sizeof d.args, "argument blocks");
    std::memcpy(out.args, d.args, sizeof d.args);
    if (name) *name = nm;
    return true;
}

int ng_time_task_device(ng_graph* g, int id, int as_executed, int reps, float* median_us, float* min_us) {
    if (!g) return NG_EINVAL;
    if (g->phase < (as_executed ? CAPTURED : BOUND)) return g->fail(NG_ESTATE, "ng_time_task_device: call %s first", as_executed ? "ng_capture" : "ng_bind");
    if (id < 0 || id >= (int)g->nodes.size() || reps <= 0 || reps > 100000 || !median_us) return g->fail(NG_EINVAL, "ng_time_task_device: bad argument");
    *median_us = 0.f;
    if (min_us) *min_us = 0.f;
    Task t = g->tasks[id];
    if (as_executed && !executed_task(g, id, g->mode, t, nullptr)) return NG_OK;
    if (!t.fn) return NG_OK;
    Runtime& rt = *g->rt;
    hipStream_t s = rt.streams[0];
    const void* fn = timed_kernel_handle(t.kid);
    if (!fn) return g->fail(NG_EINVAL, "ng_time_task_device: kernel %d has no timed variant", t.kid);
    const size_t wgs = (size_t)t.grid[0] * t.grid[1] * t.grid[2];
    if (rt.stamps_wgs < wgs) {                                     // one pair of readings per workgroup
        if (rt.stamps) (void)hipFree(rt.stamps), rt.stamps = nullptr, rt.stamps_wgs = 0;
        NG_HIP(hipMalloc(reinterpret_cast<void**>(&rt.stamps), wgs * 2 * sizeof(unsigned long long)));
        rt.stamps_wgs = wgs;
    }
    unsigned long long* stamps = rt.stamps;
    void* args[2] = {t.args, &stamps};
    std::vector<unsigned long long> h(2 * wgs);
    std::vector<float> us;
    NG_HIP(hipStreamSynchronize(s));
    for (int rep = -2; rep < reps; ++rep) {                        // two untimed launches first
        NG_HIP(hipLaunchKernel(fn, dim3(t.grid[0], t.grid[1], t.grid[2]), dim3(t.block[0], t.block[1], t.block[2]), args, t.lds_bytes, s));
        NG_HIP(hipStreamSynchronize(s));                           // solo: nothing else is in flight when the next one starts
        if (rep < 0) continue;
        NG_HIP(hipMemcpy(h.data(), rt.stamps, h.size() * sizeof(unsigned long long), hipMemcpyDeviceToHost));
        unsigned long long first = ~0ull, last = 0;
        for (size_t b = 0; b < wgs; ++b) first = std::min(first, h[2 * b]), last = std::max(last, h[2 * b + 1]);
        if (last >= first) us.push_back(0.01f * (float)(last - first));   // 100 MHz clock
    }
    if (us.empty()) return g->fail(NG_EHIP, "ng_time_task_device: the kernel left no clock readings");
    std::sort(us.begin(), us.end());
    *median_us = us[us.size() / 2];
    if (min_us) *min_us = us.front();
    return NG_OK;
}

int ng_launch_task_solo(ng_graph* g, int id, int as_executed) {
    if (!g) return NG_EINVAL;
    if (g->phase < (as_executed ? CAPTURED : BOUND)) return g->fail(NG_ESTATE, "ng_launch_task_solo: call %s first", as_executed ? "ng_capture" : "ng_bind");
    if (id < -1 || id >= (int)g->nodes.size()) return g->fail(NG_EINVAL, "ng_launch_task_solo: no node %d", id);
    hipStream_t s = g->rt->streams[0];
    if (id < 0) {
        NG_HIP(hipLaunchKernel(empty_kernel_handle(), dim3(1), dim3(64), nullptr, 0, s));
    } else {
        Task t = g->tasks[id];
        if (as_executed && !executed_task(g, id, g->mode, t, nullptr)) return NG_OK;
        if (!t.fn) return NG_OK;
        void* args[1] = {t.args};
        NG_HIP(hipLaunchKernel(t.fn, dim3(t.grid[0], t.grid[1], t.grid[2]), dim3(t.block[0], t.block[1], t.block[2]), args, t.lds_bytes, s));
    }
    NG_HIP(hipStreamSynchronize(s));
    return NG_OK;
}

const char* ng_task_kernel_executed(const ng_graph* g, int id) {
    if (!g || g->phase < CAPTURED || id < 0 || id >= (int)g->tasks.size()) return "";
    Task t;
    const char* name = "";
    return executed_task(g, id, g->mode, t, &name) ? name : "";
}

int ng_time_launch_floor(ng_graph* g, int reps, float* median_us) {
    if (!g) return NG_EINVAL;
    if (g->phase < BOUND) return g->fail(NG_ESTATE, "ng_time_launch_floor: call ng_bind first");
    if (reps <= 0 || reps > 100000 || !median_us) return g->fail(NG_EINVAL, "ng_time_launch_floor: bad argument");
    hipStream_t s = g->rt->streams[0];
    NG_HIP(hipStreamSynchronize(s));
    std::vector<float> us;
    for (int rep = -3; rep < reps; ++rep) {
        const auto t0 = std::chrono::steady_clock::now();
        NG_HIP(hipLaunchKernel(empty_kernel_handle(), dim3(1), dim3(64), nullptr, 0, s));
        NG_HIP(hipStreamSynchronize(s));
        if (rep >= 0) us.push_back(std::chrono::duration<float, std::micro>(std::chrono::steady_clock::now() - t0).count());
    }
    std::sort(us.begin(), us.end());
    *median_us = us[us.size() / 2];
    return NG_OK;
}

const char* ng_task_kernel(const ng_graph* g, int id) {
    if (!g || g->phase < BOUND || id < 0 || id >= (int)g->tasks.size()) return "";
    return g->tasks[id].name;
}

}  // extern "C"
