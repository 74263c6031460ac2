// What the launch-based replay modes launch, and the dependency edges of the multi-stream
// HIP graph. Pure host code (no HIP calls), so the edge list can be checked on a machine
// without a GPU.
//
// Nimble (arXiv 2012.02732), Section 4.1: the pre-run records the tasks in submission order
// with their streams and synchronisations, and the record is replayed as one graph launch.
// Section 4.2 / Appendix A: a plan is safe when every edge of E is ordered by FIFO order
// inside a stream or by a synchronised edge. The graph written here must carry exactly
// that order between the kernels that are actually launched.
#include <algorithm>

#include "ng_device.h"
#include "ng_internal.h"

namespace ng {

// Which tasks have no launch of their own in modes 0-3:
//   * a batch-norm / ReLU whose only input is a convolution result is applied by that
//     convolution's kernel (fused_into[v] = the convolution);
//   * a concat all of whose inputs the memory plan placed inside its result has nothing to
//     copy (fused_into[v] = v);
//   * weight updates that nothing depends on are carried out by the launch of the last such update of their stream
//     (`one_stream`: of the whole submission order; fused_into[v] = that update). A later launch is always in order
//     for an update: it already comes after every reader of its weights, and it keeps its place in the stream, so
//     the last one's launch comes after everything the earlier ones waited for;
//   * the input gradient and the parameter gradients of a batch-norm (same dy, same x) are computed by one launch, at
//     the place of whichever of the two tasks comes first on their stream (fused_into[the later one] = the earlier
//     one). Both are ready when the first one is (same inputs), each tensor has its buffer to itself, and the later
//     task's place in the stream is behind the launch, so whatever follows it in the stream or waits for its event
//     is ordered after the launch.
// Everything else: -1. `tasks` needs the kernel ids only (a dry task table will do).
void decide_launch_fusion(const ng_graph* g, const std::vector<Task>& tasks, bool fuse, bool one_stream, std::vector<int>& fused_into) {
    const int n = (int)g->nodes.size();
    fused_into.assign(n, -1);
    // not under a memory plan with reuse over time: there the batch-norm's buffer may still hold the
    // convolution's own input when the convolution runs
    if (!fuse || g->memory_reuse) return;
    std::vector<char> has_epilogue(n, 0);
    for (int v = 0; v < n; ++v) {
        const Node& nd = g->nodes[v];
        if ((nd.op != NG_OP_BN_ACT && nd.op != NG_OP_RELU) || nd.preds.size() != 1) continue;
        const int u = nd.preds[0];
        // a graph that trains: the conv1x1 kernel that streams the pixels applies a batch-norm from its raw parameters
        const bool raw = nd.op == NG_OP_BN_ACT && tasks[v].kid == KID_BN_RAW && tasks[u].kid == KID_PW_PX_FWD;
        if (!tasks[u].fn || !(has_bn_epilogue(tasks[u].kid) || raw) || has_epilogue[u] || !(g->nodes[u].out == nd.out)) continue;
        has_epilogue[u] = 1;
        fused_into[v] = u;
    }
    for (int v = 0; v < n && !g->alias_of.empty(); ++v) {
        const Node& nd = g->nodes[v];
        if (nd.op != NG_OP_CONCAT) continue;
        bool in_place = true;
        for (int u : nd.preds) in_place = in_place && g->alias_of[u] == v && tasks[u].fn;
        if (in_place) fused_into[v] = v;
    }
    const Schedule& sc = g->sched;
    // batch-norm backward: input gradient and parameter gradients of the same (dy, x) are two walks over the same data;
    // whichever of the two comes first on their common stream computes both
    std::vector<int> pos(n, 0);
    for (int i = 0; i < (int)sc.order.size(); ++i) pos[sc.order[i]] = i;
    for (int d = 0; d < n; ++d) {
        const Node& nd = g->nodes[d];
        if (nd.op != NG_OP_BN_ACT_DGRAD || tasks[d].kid != KID_BN_DGRAD) continue;
        for (int w = 0; w < n; ++w) {
            const Node& nw = g->nodes[w];
            if (nw.op != NG_OP_BN_ACT_WGRAD || tasks[w].kid != KID_BN_WGRAD || fused_into[w] >= 0 || nw.preds != nd.preds ||
                nw.weights != nd.weights || nw.p.relu != nd.p.relu || nw.p.eps != nd.p.eps)
                continue;
            if (!one_stream && sc.stream_of[w] != sc.stream_of[d]) continue;
            bool taken = false;                                   // w already computes another node's input gradient
            for (int v = 0; v < n; ++v) taken = taken || fused_into[v] == w;
            if (taken) continue;
            if (pos[d] < pos[w]) fused_into[w] = d; else fused_into[d] = w;
            break;
        }
    }
    // the input gradient and the weight gradient of a depthwise or 1 x 1 convolution read the same dy and are each bound by
    // latency when alone: one launch with their workgroups interleaved, at the place of whichever comes first - if
    // everything the later one reads is complete by then (its inputs all come before the earlier one on the stream)
    for (int d = 0; d < n; ++d) {
        const Node& nd = g->nodes[d];
        if ((nd.op != NG_OP_DWCONV_DGRAD && nd.op != NG_OP_CONV1X1_DGRAD) || !tasks[d].fn || fused_into[d] >= 0) continue;
        for (int w = 0; w < n; ++w) {
            const Node& nw = g->nodes[w];
            if (nw.op != (nd.op == NG_OP_DWCONV_DGRAD ? NG_OP_DWCONV_WGRAD : NG_OP_CONV1X1_WGRAD) || !tasks[w].fn || fused_into[w] >= 0 ||
                nw.preds.empty() || nd.preds.empty() || nw.preds[0] != nd.preds[0] || !can_pair(tasks[d].kid, tasks[w].kid))
                continue;
            if (!one_stream && sc.stream_of[w] != sc.stream_of[d]) continue;
            const int early = pos[d] < pos[w] ? d : w, late = early == d ? w : d;
            bool ready = true, taken = false;
            for (int u : g->nodes[late].preds) ready = ready && pos[u] < pos[early] && (one_stream || sc.stream_of[u] == sc.stream_of[early]);
            for (int v = 0; v < n; ++v) taken = taken || fused_into[v] == w || fused_into[v] == d;
            if (!ready || taken) continue;
            fused_into[late] = early;
            break;
        }
    }
    std::vector<char> is_read(n, 0);
    for (int v = 0; v < n; ++v)
        for (int u : g->nodes[v].preds) is_read[u] = 1;
    std::vector<int> last_update(one_stream ? 1 : sc.n_streams, -1);
    for (auto it = sc.order.rbegin(); it != sc.order.rend(); ++it) {
        const int v = *it;
        if (g->nodes[v].op != NG_OP_SGD_UPDATE || tasks[v].kid != KID_SGD || is_read[v]) continue;
        int& last = last_update[one_stream ? 0 : sc.stream_of[v]];
        if (last < 0) last = v;
        else fused_into[v] = last;
    }
}

// The multi-stream graph: one kernel node per launched task, in submission order; a node
// depends on the previous task of its stream (FIFO order within a stream) and on the
// producer of every planned event wait (Lambda). A task without a launch of its own keeps
// its place in its stream and its events: whatever depends on it depends on everything it
// depended on. Fork / join scaffolding of a capture carries no dependency and has no
// counterpart here.
void build_launch_graph(const ng_graph* g, const std::vector<Task>& tasks, const std::vector<int>& fused_into, LaunchGraph& out) {
    const Schedule& sc = g->sched;
    const int n = (int)g->nodes.size();
    out.nodes.clear();
    out.deps.clear();
    std::vector<std::vector<int>> stands_for(n);       // launched tasks a dependency on v amounts to
    std::vector<int> last_on_stream(sc.n_streams, -1);
    for (int v : sc.order) {
        const bool launched = tasks[v].fn != nullptr && fused_into[v] < 0;
        if (!launched && fused_into[v] < 0) continue;  // network input: no task, nothing to order
        const int st = sc.stream_of[v];
        std::vector<int> deps;
        auto depend_on = [&](int u) {
            for (int d : stands_for[u])
                if (std::find(deps.begin(), deps.end(), d) == deps.end()) deps.push_back(d);
        };
        if (last_on_stream[st] >= 0) depend_on(last_on_stream[st]);
        for (int u : sc.waits[v]) depend_on(u);
        last_on_stream[st] = v;
        if (!launched) {
            stands_for[v] = deps;
            continue;
        }
        stands_for[v].assign(1, v);
        out.nodes.push_back(v);
        out.deps.push_back(std::move(deps));
    }
}

}  // namespace ng

using namespace ng;

namespace {
// The task table as far as the host needs it (kernel ids), built against fake addresses
// when nothing is bound yet.
struct TaskView {
    ng_graph* g;
    std::vector<Task> saved;
    bool dry = false;
    int rc = NG_OK;
    explicit TaskView(ng_graph* graph) : g(graph) {
        if (g->phase >= BOUND) return;
        dry = true;
        saved.swap(g->tasks);
        g->dry_run = true;
        g->tasks.assign(g->nodes.size(), Task());
        char* fake_arena = reinterpret_cast<char*>(0x100000000ull);
        static float fake_constants;
        for (int v = 0; v < (int)g->nodes.size() && rc == NG_OK; ++v) rc = build_task(g, v, fake_arena, &fake_constants, g->tasks[v]);
    }
    ~TaskView() {
        if (!dry) return;
        g->dry_run = false;
        g->tasks.swap(saved);
    }
};
}  // namespace

extern "C" int ng_get_graph_edges(ng_graph* g, int fuse, int* launched_by, int* n_edges, int* src, int* dst, int max_edges) {
    if (!g) return NG_EINVAL;
    if (g->phase < PLANNED) return g->fail(NG_ESTATE, "ng_get_graph_edges: call ng_plan_memory first");
    if (max_edges < 0 || (max_edges > 0 && (!src || !dst))) return g->fail(NG_EINVAL, "ng_get_graph_edges: bad edge arrays");
    TaskView view(g);
    if (view.rc != NG_OK) return view.rc;
    std::vector<int> fused_into;
    decide_launch_fusion(g, g->tasks, fuse != 0, fuse == 2, fused_into);
    LaunchGraph lg;
    if (fuse == 2) {                                           // one stream: every launch follows the one before it
        for (int v : g->sched.order) {
            if (!g->tasks[v].fn || fused_into[v] >= 0) continue;
            lg.deps.push_back(lg.nodes.empty() ? std::vector<int>() : std::vector<int>(1, lg.nodes.back()));
            lg.nodes.push_back(v);
        }
    } else {
        build_launch_graph(g, g->tasks, fused_into, lg);
    }
    const int n = (int)g->nodes.size();
    if (launched_by)
        for (int v = 0; v < n; ++v)
            launched_by[v] = !g->tasks[v].fn ? -1 : fused_into[v] == v ? -2 : fused_into[v] >= 0 ? fused_into[v] : v;
    int count = 0;
    for (size_t i = 0; i < lg.nodes.size(); ++i)
        for (int d : lg.deps[i]) {
            if (count < max_edges) src[count] = d, dst[count] = lg.nodes[i];
            ++count;
        }
    if (n_edges) *n_edges = count;
    if (count > max_edges && max_edges > 0) return g->fail(NG_ENOMEM, "ng_get_graph_edges: %d edges, room for %d", count, max_edges);
    return NG_OK;
}

extern "C" const char* ng_planned_task_kernel(ng_graph* g, int id) {
    if (!g) return nullptr;
    if (g->phase < PLANNED) return g->fail(NG_ESTATE, "ng_planned_task_kernel: call ng_plan_memory first"), nullptr;
    if (id < 0 || id >= (int)g->nodes.size()) return g->fail(NG_EINVAL, "ng_planned_task_kernel: no node %d", id), nullptr;
    TaskView view(g);
    if (view.rc != NG_OK) return nullptr;
    const char* name = g->tasks[id].name;
    return name ? name : "";
}
