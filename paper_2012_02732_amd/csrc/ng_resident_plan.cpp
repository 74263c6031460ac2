// Host-side planner of the device-resident replay: turns the task schedule into one static
// task list per persistent workgroup. Pure host code (no HIP calls), so it is testable
// without a GPU.
//
// Nimble (arXiv 2012.02732) fixes *everything* about a run ahead of time (Section 4.1) and
// lets independent operators run side by side on different streams (Section 4.2). Here the
// same two ideas are applied one level further down: which workgroup executes which tile of
// which task, and in what order, is also decided ahead of time.
//
//   * A stream lives on one XCD (workgroup w of a 1-D grid runs on XCD w mod 8), so the
//     tensors that flow along a stream stay in that XCD's L2. Streams are placed heaviest
//     first on the XCD with the least work so far.
//   * The workgroups of an XCD are shared by the streams placed on it. Tasks are taken in
//     the order in which their inputs are expected to be ready and each is given the workgroups
//     of its XCD that a simple cost model expects to be free first - classic list
//     scheduling - trying 1..4 rounds of tiles per workgroup and keeping the earliest
//     expected finish. Independent tasks therefore land on different workgroups and overlap;
//     dependent ones reuse the workgroups that just finished their producer.
//   * A task with more tiles than one XCD has workgroups may be spread over every participating
//     XCD when that is expected to pay for the longer way its data then takes.
//   * An elementwise task can take over the tile partition and the workgroups of the E' parent
//     on its stream; that wait is then dropped (tile i needs only what the same workgroup wrote).
//   * Every workgroup's list is a subsequence of one topological order (the order in which the
//     planner placed the tasks) and a task waits only for earlier tasks, so with all
//     workgroups resident no wait can depend on itself.
//   * Otherwise a task waits for all of its E' parents (FIFO order inside a stream does not
//     order two workgroups): through a counter in the XCD's L2 when producer and consumer share
//     the XCD, through a device-scope counter when not. Whether a tensor is stored and loaded
//     with device-scope accesses is decided from *all* direct readers (edges of E): a reader on
//     another XCD reads the tensor itself, even when it only waits for an intermediate task.
//   * The constants of the cost model that decide between plans of similar expected length
//     (PlanKnobs) come with the call: the runtime plans under several settings of them
//     (plan_setting) and keeps the plan that replays fastest, and can pass per-task correction
//     factors measured in a traced replay.
#include <algorithm>
#include <functional>
#include <cstdlib>
#include <cstring>
#include <numeric>
#include <queue>
#include <tuple>

#include "ng_device.h"
#include "ng_internal.h"

namespace ng {

namespace {

constexpr double kLocalUs = 0.1;      // hand-over inside one workgroup: one barrier
constexpr double kFusedUs = 0.05;     // a batch-norm applied in the convolution's registers: a few instructions, one more store

// Expected time of one round of a task, in microseconds, when `subs` sub-blocks of a
// workgroup take a tile each: a latency part that does not depend on how many tiles share
// the compute unit (address set-up, one trip to memory and back for the loads, one for the
// stores) plus a throughput part per tile (load issue and data return of the compute
// unit's one memory pipeline, matrix-core time of wavefronts that share a SIMD). Figures
// from traces of the resident kernel; the planner only needs them to be ordered sensibly.
double tile_round_us(const ng_graph* g, int v, int kid_any, int subs) {
    const int kid = plain_variant(kid_any);
    const Node& nd = g->nodes[v];
    const double cin = nd.preds.empty() ? 0.0 : (double)g->nodes[nd.preds[0]].out.c;
    double base = 1.0, per_tile = 0.1;
    switch (kid) {
        case KID_BN: case KID_BN_V4: case KID_BN_R64: case KID_BN_R16: base = 1.2, per_tile = 0.15; break;
        case KID_ADD: case KID_ADD_V4: case KID_ADD_R64: case KID_ADD_R16: base = 0.9, per_tile = 0.1; break;
        case KID_CONCAT: case KID_CONCAT_V4: base = 1.6, per_tile = 0.2; break;
        case KID_POOL: base = 1.6, per_tile = 0.25; break;
        case KID_POOL_ROW_S1: case KID_POOL_ROW_S2: base = 1.8, per_tile = 0.5; break;
        case KID_POOL_P4: case KID_DW_K3S1_P4: base = 1.9, per_tile = 0.6; break;
        case KID_DW_K3S1: case KID_DW_K3S2: base = 1.5, per_tile = 0.25; break;
        case KID_DW_K5S1: case KID_DW_K5S2: base = 2.0, per_tile = 0.7; break;
        case KID_GAP: base = 1.0, per_tile = 0.1; break;
        case KID_FC_GEMV: base = 1.0 + 0.001 * cin * (double)nd.out.n, per_tile = 0.2; break;
        case KID_PW_D4: case KID_PW_D8: case KID_PW_D16: base = 1.3, per_tile = 0.4 + 0.008 * cin; break;
        case KID_PW_64: base = 1.5, per_tile = 0.025 * cin; break;
        case KID_PW_P64: base = 1.5, per_tile = 0.02 * cin; break;
        case KID_PW_P32: base = 1.5, per_tile = 0.012 * cin; break;
        case KID_PW_V1: case KID_PW_V2: case KID_PW_V3: case KID_PW_V4: {
            const PwArgs* a = reinterpret_cast<const PwArgs*>(g->tasks[v].args);
            base = 1.3, per_tile = 0.3 * (a->ksteps / 4);           // per group of 4 k-steps and wavefront: 5 128-bit loads, 16 MFMAs
            break;
        }
        case KID_PW_S1: case KID_PW_S2: case KID_PW_S3: case KID_PW_S4: {
            const PwArgs* a = reinterpret_cast<const PwArgs*>(g->tasks[v].args);
            base = 1.6, per_tile = 0.12 * (a->ksteps / 4);
            break;
        }
        case KID_C3_T16S1: case KID_C3_T16S2: case KID_C3_T8S1: case KID_C3_T8S2: base = 1.0, per_tile = 0.375 * cin; break;
        case KID_C3_M1: case KID_C3_M2: case KID_C3_M3: case KID_C3_M4: {
            const C3Args* a = reinterpret_cast<const C3Args*>(g->tasks[v].args);
            base = 1.8, per_tile = 0.2 * (a->groups / 4);
            break;
        }
        case KID_C3_L32: base = 2.0, per_tile = 0.14 * cin; break;     // 9 Cin / 4 k-steps of 4 MFMAs per wavefront, plus the slice fills
        case KID_C3_L64: base = 2.0, per_tile = 0.16 * cin; break;
        case KID_C3_P64: case KID_C3_Q64: case KID_C3_Q32: base = 2.5, per_tile = 0.3 * cin; break;   // 9 Cin / 16 slices of 16 (64 x 64) MFMAs per wavefront
        case KID_C3_P96: base = 2.5, per_tile = 0.45 * cin; break;
        case KID_C3_Q128: base = 2.5, per_tile = 0.6 * cin; break;
        case KID_PW_PX_FWD: case KID_PW_PX_DGRAD: base = 2.0, per_tile = 0.6; break;
        case KID_SMALL_GEMM: base = 2.5, per_tile = 0.3; break;
        case KID_GEMM_PW_FWD: case KID_GEMM_PW_DGRAD: case KID_GEMM_PW_WGRAD: case KID_GEMM_C3_FWD: case KID_GEMM_C3_DGRAD:
        case KID_GEMM_C3_WGRAD: {
            const GemmArgs* a = reinterpret_cast<const GemmArgs*>(g->tasks[v].args);
            base = 2.0, per_tile = 0.04 * a->k_per_split;             // per K slice of 16: gathered loads, LDS fill, 16 MFMAs per wavefront
            break;
        }
        case KID_PW_WGRAD_PX: case KID_PW_WGRAD_PX2: case KID_C3_WGRAD_PX: case KID_C3_WGRAD_PX2: {
            const GemmArgs* a = reinterpret_cast<const GemmArgs*>(g->tasks[v].args);
            base = 4.0, per_tile = ((kid == KID_PW_WGRAD_PX || kid == KID_C3_WGRAD_PX) ? 0.001 : 0.002) * a->k_per_split;   // 4 or 16 MFMAs per wavefront and slice of 16 pixels, four wavefronts side by side; then the sum
            break;
        }
        case KID_BN_RAW: case KID_BN_DGRAD: case KID_RELU_DGRAD: case KID_GAP_DGRAD: case KID_SLICE_PAD: case KID_SGD: base = 1.2, per_tile = 0.15; break;
        case KID_DW_DGRAD: case KID_POOL_DGRAD: base = 2.0, per_tile = 0.7; break;
        case KID_POOL_DGRAD_LDS: case KID_DW_DGRAD_LDS: case KID_DW_LDS: base = 2.5, per_tile = 1.0; break;
        case KID_BN_WGRAD: case KID_CHANNEL_SUM: {
            double count = (double)g->nodes[nd.preds[0]].out.elems() / std::max<double>(1.0, (double)g->nodes[nd.preds[0]].out.c);
            if (kid == KID_BN_WGRAD) count /= std::max(1, reinterpret_cast<const BnRawArgs*>(g->tasks[v].args)->chunks);   // a channel's images are split over workgroups
            base = 1.5 + 0.00002 * count * 256.0 / kBlock, per_tile = 0.00003 * count;   // one workgroup walks a whole channel
            break;
        }
        case KID_DW_WGRAD: {                                           // one workgroup per (channel, chunk of images)
            const DwGradArgs* a = reinterpret_cast<const DwGradArgs*>(g->tasks[v].args);
            const double count = (double)g->nodes[nd.preds[0]].out.h * (double)g->nodes[nd.preds[0]].out.w * ((a->N + a->chunks - 1) / std::max(1, a->chunks));
            base = 2.5, per_tile = 0.0005 * count;
            break;
        }
        default: break;
    }
    return base + per_tile * subs;
}

// The kernel variant of an elementwise task that uses partition `part` (KID_NONE if there is
// none), and the number of tiles that partition has.
int variant_for(const ng_graph* g, int v, int part, long* ntiles) {
    const Node& nd = g->nodes[v];
    const Shape& o = nd.out;
    const long total = o.elems(), hw = o.h * o.w, cols = o.n * hw;
    const bool bn = nd.op == NG_OP_BN_ACT || nd.op == NG_OP_RELU, add = nd.op == NG_OP_ADD_N;
    if (!bn && !add) return KID_NONE;
    switch (part) {
        case PART_L256: *ntiles = (total + kBlock - 1) / kBlock; return bn ? KID_BN : KID_ADD;
        case PART_L1024:
            if ((bn && hw % 4 != 0) || (add && total % 4 != 0)) return KID_NONE;
            *ntiles = (total / 4 + kBlock - 1) / kBlock;
            return bn ? KID_BN_V4 : KID_ADD_V4;
        case PART_R64:
            if (hw % 4 != 0) return KID_NONE;
            *ntiles = ((o.c + 15) / 16) * ((cols + 63) / 64);
            return bn ? KID_BN_R64 : KID_ADD_R64;
        case PART_R16: *ntiles = ((o.c + 15) / 16) * ((cols + 15) / 16); return bn ? KID_BN_R16 : KID_ADD_R16;
        default: return KID_NONE;
    }
}

struct Sim {
    std::vector<std::vector<DevEntry>> lists;
    std::vector<unsigned> parts;
    std::vector<unsigned> signals;   // increments of the device-scope counter per replay: participants, or XCDs used (two-level)
    std::vector<int> xcd;
    std::vector<int> kid;            // kernel variant chosen for the resident replay
    std::vector<long> ntiles;        // its tile count
    std::vector<int> subs;           // sub-blocks per workgroup that take a tile each
    std::vector<int> order;          // tasks in the order they were placed: every workgroup's list follows it
    std::vector<int> local_parent;   // E' parent whose completion this task does not wait for (same workgroups, same tiles), or -1
    std::vector<int> fused_into;     // convolution whose tiles also produce this (batch-norm / ReLU / add_n) task's result, or -1
    std::vector<char> elided;        // concat whose inputs were all produced in place: no work, no entries
    std::vector<double> model_run;   // what the model expects between a task's last wait and its last store
    double makespan = 0;
};

void simulate(const ng_graph* g, int n_wg, int nx, const PlanKnobs& knobs, Sim& out) {
    const double kSyncNearUs = knobs.sync_near_us, kSyncFarUs = knobs.sync_far_us, kSpreadPenaltyUs = knobs.spread_penalty_us;
    const double kPublishUs = knobs.publish_us, kFarRunFactor = knobs.far_run_factor;
    // the model's round time, corrected by what a traced replay measured for this task (if anything)
    auto round_us = [&](int v, int kid, int subs) {
        return tile_round_us(g, v, kid, subs) * (knobs.task_scale.empty() ? 1.0 : knobs.task_scale[v]);
    };
    const Schedule& sc = g->sched;
    const int n = (int)g->nodes.size();
    const int per_xcd = n_wg / 8;
    const bool debug = knob("NG_PLAN_DEBUG") != nullptr;
    // (under a memory plan with reuse over time a task's result may live where its producer's own input still is: every task
    // then waits for the completion of all its producers, and no task runs inside another task's tiles)
    const bool allow_local = knob("NG_NO_LOCAL") == nullptr && !g->memory_reuse;

    // the planner counts work in units of `subs` tiles: what one workgroup does in one round
    auto units_for = [&](long ntiles, int subs) { return (ntiles + subs - 1) / subs; };
    std::vector<long> stream_work(sc.n_streams, 0);
    for (int v = 0; v < n; ++v) stream_work[sc.stream_of[v]] += units_for(g->tasks[v].ntiles, kSubs);
    std::vector<int> by_work(sc.n_streams);
    std::iota(by_work.begin(), by_work.end(), 0);
    std::stable_sort(by_work.begin(), by_work.end(), [&](int a, int b) { return stream_work[a] > stream_work[b]; });
    std::vector<long> xcd_work(nx, 0);
    std::vector<int> xcd_count(nx, 0), stream_xcd(sc.n_streams, 0);
    for (int st : by_work) {
        int best = 0;
        for (int x = 1; x < nx; ++x)
            if (xcd_work[x] < xcd_work[best] || (xcd_work[x] == xcd_work[best] && xcd_count[x] < xcd_count[best])) best = x;
        stream_xcd[st] = best;
        ++xcd_count[best];
        xcd_work[best] += std::max<long>(stream_work[st], 1);
    }

    out.lists.assign(n_wg, {});
    out.parts.assign(n, 0);
    out.signals.assign(n, 0);
    out.xcd.assign(n, -1);
    out.kid.assign(n, KID_NONE);
    out.ntiles.assign(n, 0);
    out.subs.assign(n, kSubs);
    out.local_parent.assign(n, -1);
    out.fused_into.assign(n, -1);
    out.elided.assign(n, 0);
    out.model_run.assign(n, 0.0);
    const bool allow_elide = knob("NG_NO_ELIDE") == nullptr;
    const bool allow_fuse = knob("NG_NO_FUSE") == nullptr && !g->memory_reuse;
    std::vector<double> free_at(n_wg, 0.0), finish(n, 0.0);
    std::vector<std::vector<int>> parents(n), wgs(n);
    for (auto& e : sc.meg) parents[e.second].push_back(e.first);

    // Tasks are taken in the order in which the model expects their inputs to be ready (ties:
    // the longer remaining path first) - a topological order like ascending id, but one that
    // does not make a workgroup sit in front of a task of a slow branch while a task of
    // another stream further down its list could already run.
    std::vector<std::vector<int>> children(n);
    std::vector<int> waiting(n, 0);
    for (auto& e : sc.meg)
        if (g->tasks[e.first].fn && g->tasks[e.second].fn) children[e.first].push_back(e.second), ++waiting[e.second];
    std::vector<double> tail(n, 0.0);
    for (int v = n - 1; v >= 0; --v) {
        if (!g->tasks[v].fn) continue;
        double longest = 0;
        for (int c : children[v]) longest = std::max(longest, tail[c]);
        tail[v] = longest + round_us(v, g->tasks[v].kid, kSubs) + kSyncNearUs;
    }
    auto ready_time = [&](int v) {                              // all parents placed: when the last of them is visible
        const int home = stream_xcd[sc.stream_of[v]];
        double ready = 0;
        for (int u : parents[v]) {
            if (!g->tasks[u].fn) continue;
            const bool far = nx > 1 && (out.xcd[u] < 0 || out.xcd[u] != home);
            ready = std::max(ready, finish[u] + (far ? kSyncFarUs : 0.0));
        }
        return ready;
    };
    typedef std::tuple<double, double, int> Key;                // (ready time, -tail, id): smallest first
    std::priority_queue<Key, std::vector<Key>, std::greater<Key>> open;
    for (int v = 0; v < n; ++v)
        if (g->tasks[v].fn && waiting[v] == 0) open.push(Key(0.0, -tail[v], v));
    out.order.clear();
    std::vector<char> fused_child(n, 0);                        // the convolution already carries a batch-norm epilogue
    std::vector<char> add_child(n, 0);                          // ... an add_n epilogue
    std::vector<int> placed_at(n, -1);                          // position in out.order
    const bool allow_fuse_add = allow_fuse && knob("NG_NO_FUSE_ADD") == nullptr;

    while (!open.empty()) {
        const int v = std::get<2>(open.top());
        open.pop();
        placed_at[v] = (int)out.order.size();
        out.order.push_back(v);
        const Task& t = g->tasks[v];
        const int home = stream_xcd[sc.stream_of[v]];
        out.kid[v] = t.kid;
        out.ntiles[v] = t.ntiles;
        // a windowed task that would need more than `p4_rounds` rounds on its stream's workgroups gets 4
        // outputs per thread (4 x the index arithmetic in one round: pays off only from there)
        const int p4_rounds = (int)knob_int("NG_P4_ROUNDS", 1, 1 << 20, knobs.p4_rounds);
        if (units_for(t.ntiles, kSubs) > p4_rounds * per_xcd && (t.kid == KID_POOL || t.kid == KID_DW_K3S1) &&
            !knob("NG_NO_P4")) {
            out.kid[v] = t.kid == KID_POOL ? KID_POOL_P4 : KID_DW_K3S1_P4;
            out.ntiles[v] = (g->nodes[v].out.elems() + 4 * kBlock - 1) / (4 * kBlock);
        }
        // A concat whose inputs the memory plan placed inside its result has nothing to copy: it gets
        // no entries, and whoever waits for it waits for its producers instead.
        if (allow_elide && g->nodes[v].op == NG_OP_CONCAT && !g->alias_of.empty()) {
            bool in_place = true;
            for (int u : g->nodes[v].preds) in_place = in_place && g->alias_of[u] == v && g->tasks[u].fn;
            for (int c : children[v]) in_place = in_place && parents[c].size() - 1 + parents[v].size() <= (size_t)NG_MAX_PREDS;
            if (in_place) {
                out.elided[v] = 1;
                out.kid[v] = KID_NONE;                      // nobody can take over its partition
                out.ntiles[v] = 0;
                int common = -2;                            // the XCD all producers ran on, else -1 (treated like a spread task)
                double done = 0;
                for (int u : g->nodes[v].preds) common = common == -2 ? out.xcd[u] : (common == out.xcd[u] ? common : -1);
                for (int u : parents[v]) done = std::max(done, finish[u]);
                out.xcd[v] = common;
                finish[v] = done;
                if (debug) fprintf(stderr, "PLAN nx=%d v=%d concat in place, xcd=%d finish=%.2f\n", nx, v, common, done);
                for (int c : children[v])
                    if (--waiting[c] == 0) open.push(Key(ready_time(c), -tail[c], c));
                continue;
            }
        }
        // A batch-norm / ReLU task whose only producer is a convolution is not run at all: the
        // convolution's tiles apply it to their results before they store them (same values, same
        // arithmetic), and whoever waits for this task waits for the convolution.
        if (allow_fuse && allow_local && (g->nodes[v].op == NG_OP_BN_ACT || g->nodes[v].op == NG_OP_RELU) &&
            parents[v].size() == 1 && g->nodes[v].preds.size() == 1 && parents[v][0] == g->nodes[v].preds[0]) {
            const int u = parents[v][0];
            if (g->tasks[u].fn && has_bn_epilogue(out.kid[u]) && !fused_child[u] && g->nodes[u].out == g->nodes[v].out) {
                fused_child[u] = 1;
                out.fused_into[v] = u;
                out.local_parent[v] = u;
                // an elementwise task behind v may still take over the tile grid (16-row kernels only)
                long nt = 0;
                const int kid = variant_for(g, v, partition_of(out.kid[u]), &nt);
                out.kid[v] = kid != KID_NONE && nt == out.ntiles[u] ? kid : KID_NONE;
                out.ntiles[v] = out.kid[v] != KID_NONE ? nt : 0;
                out.subs[v] = out.subs[u];
                out.xcd[v] = out.xcd[u];
                wgs[v] = wgs[u];
                out.parts[v] = out.parts[u];
                out.signals[v] = out.signals[u];
                finish[v] = finish[u] + kFusedUs;
                out.makespan = std::max(out.makespan, finish[v]);
                if (debug) fprintf(stderr, "PLAN nx=%d v=%d fused into %d finish=%.2f\n", nx, v, u, finish[v]);
                for (int c : children[v])
                    if (--waiting[c] == 0) open.push(Key(ready_time(c), -tail[c], c));
                continue;
            }
        }
        // An add_n with one operand that is such a convolution result (raw or batch-normed) and is
        // read by nobody else goes the same way: the convolution's tiles wait for the producers
        // of the other operands once their own sums are done, add and store. Those producers
        // must come before the convolution in the common order of the lists (waits only point
        // backwards), which is the case when the convolution is the later branch - the case
        // in which the fused add_n saves a hand-over on the critical path.
        if (allow_fuse_add && allow_local && g->nodes[v].op == NG_OP_ADD_N && g->nodes[v].preds.size() >= 2 &&
            g->nodes[v].preds.size() <= (size_t)kEpilogueAddMax) {
            const std::vector<int>& preds = g->nodes[v].preds;
            int host = -1, via = -1;
            // first choice: a host on the XCD of the add_n's own stream, where its readers most likely are
            const int far_host = (int)knob_int("NG_FUSE_ADD_FAR", 0, 1, 1);
            for (int pass = 0; pass < 1 + far_host && host < 0; ++pass)
            for (int w : parents[v]) {
                const int u = out.fused_into[w] >= 0 ? out.fused_into[w] : w;
                if (!g->tasks[u].fn || add_child[u]) continue;
                if ((out.xcd[u] == (nx == 1 ? 0 : home)) != (pass == 0)) continue;
                if (g->nodes[w].op == NG_OP_ADD_N) continue;                               // w must be the convolution or its batch-norm
                if (add_variant(out.kid[u]) == KID_NONE || (w == u && fused_child[u])) continue;   // a 16-row convolution or a pool
                // nobody else reads the convolution or its batch-norm, and the value is one operand exactly once
                if (children[u].size() != 1 || children[w].size() != 1 || children[w][0] != v) continue;
                if (std::count(preds.begin(), preds.end(), w) != 1 || (w != u && std::count(preds.begin(), preds.end(), u) != 0)) continue;
                long nt = 0;
                if (!(g->nodes[u].out == g->nodes[v].out) || variant_for(g, v, partition_of(out.kid[u]), &nt) == KID_NONE || nt != out.ntiles[u]) continue;
                bool before = true;
                for (int p : parents[v]) {
                    if (p == w || !g->tasks[p].fn) continue;
                    const int src = out.fused_into[p] >= 0 ? out.fused_into[p] : p;      // whose counter the late wait watches
                    before = before && src != u && !out.elided[src] && placed_at[src] >= 0 && placed_at[src] < placed_at[u];
                }
                if (!before || parents[u].size() + parents[v].size() - 1 > (size_t)NG_MAX_PREDS) continue;
                host = u, via = w;
                break;
            }
            if (host >= 0) {
                long nt = 0;
                add_child[host] = 1;
                out.kid[host] = add_variant(out.kid[host]);          // the kernel variant that has the add_n at its end
                out.fused_into[v] = host;
                out.local_parent[v] = via;
                out.kid[v] = variant_for(g, v, partition_of(out.kid[host]), &nt);
                out.ntiles[v] = nt;
                out.subs[v] = out.subs[host];
                out.xcd[v] = out.xcd[host];
                wgs[v] = wgs[host];
                out.parts[v] = out.parts[host];
                out.signals[v] = out.signals[host];
                double ready = finish[host];
                for (int p : parents[v]) {
                    if (p == via || !g->tasks[p].fn) continue;
                    const bool far = out.xcd[p] < 0 || out.xcd[host] < 0 || out.xcd[p] != out.xcd[host] || g->resident_all_far;
                    ready = std::max(ready, finish[p] + kSyncNearUs + (far ? kSyncFarUs : 0.0));
                }
                finish[v] = ready + kFusedUs;
                if (finish[v] > finish[host] + kFusedUs)                 // the convolution's workgroups sit in the late wait
                    for (int w : wgs[host]) free_at[w] = std::max(free_at[w], finish[v] + kPublishUs);
                out.makespan = std::max(out.makespan, finish[v]);
                if (debug) fprintf(stderr, "PLAN nx=%d v=%d add fused into %d via %d finish=%.2f\n", nx, v, host, via, finish[v]);
                for (int c : children[v])
                    if (--waiting[c] == 0) open.push(Key(ready_time(c), -tail[c], c));
                continue;
            }
        }
        const int kid0 = out.kid[v];                        // before a possible change of partition below
        const long ntiles0 = out.ntiles[v];
        // Two placements are compared: on the XCD of the task's stream (inputs and outputs
        // stay in that L2 when the neighbours are there too), or spread over every
        // participating XCD (more workgroups, but everything the task touches goes through
        // the memory side, and so does whatever reads its result).
        auto ready_at = [&](int xcd_v, int skip) {
            double ready = 0;
            for (int u : parents[v]) {
                if (!g->tasks[u].fn || u == skip) continue;
                const bool far = out.xcd[u] < 0 || xcd_v < 0 || out.xcd[u] != xcd_v || g->resident_all_far;
                ready = std::max(ready, finish[u] + (far ? kSyncFarUs : 0.0));
            }
            return ready;
        };
        // only the matrix kernels keep a compute unit's memory pipeline busy enough to be worth
        // spreading one tile per workgroup; for the others fewer participants is what counts
        const bool heavy = is_matrix_kernel(kid0);
        struct Placement {
            double finish = 1e300, ready = 0;
            int p = 1, subs = kSubs;
            std::vector<int> cand;
        };
        // where = -1: every participating XCD; otherwise that XCD
        auto place = [&](int where) {
            Placement pl;
            const bool spread = where < 0;
            for (int w = 0; w < n_wg; ++w) {
                const int x = w % 8;
                if (x < nx && (spread || x == where)) pl.cand.push_back(w);
            }
            pl.ready = ready_at(nx == 1 ? 0 : where, -1);
            // do this task's loads go through the memory side? (some direct input lives elsewhere)
            bool far_loads = spread;
            for (int u : g->nodes[v].preds)
                if (g->tasks[u].fn && nx > 1 && (out.xcd[u] < 0 || out.xcd[u] != where)) far_loads = true;
            // workgroups in the order they become available for this task
            std::stable_sort(pl.cand.begin(), pl.cand.end(), [&](int a, int b) { return free_at[a] < free_at[b]; });
            for (int subs = kSubs; subs >= (heavy ? 1 : kSubs); --subs) {
                const long units = units_for(ntiles0, subs);
                const double cost = round_us(v, kid0, subs) * (far_loads ? kFarRunFactor : 1.0);
                for (int rounds = 1; rounds <= 4; ++rounds) {
                    const int p = (int)std::min<long>((units + rounds - 1) / rounds, (long)pl.cand.size());
                    const long r = (units + p - 1) / p;
                    const double f = std::max(pl.ready, free_at[pl.cand[p - 1]]) + r * cost + kSyncNearUs;
                    // same finish: fewer participants (fewer completions to collect, less skew)
                    if (f < pl.finish - 1e-9 || (f < pl.finish + 1e-9 && p < pl.p)) pl.finish = f, pl.p = p, pl.subs = subs;
                }
            }
            return pl;
        };
        const int where = nx == 1 ? 0 : home;
        Placement chosen = place(where);
        bool wide = false;
        if (nx > 1 && units_for(ntiles0, kSubs) > per_xcd) {
            Placement spread = place(-1);
            // what reads the result pays for the longer way too, unless nothing can run beside this task anyway
            if (spread.finish + (sc.solo[v] ? 0.0 : kSpreadPenaltyUs) < chosen.finish) chosen = std::move(spread), wide = true;
        }
        out.xcd[v] = nx == 1 ? 0 : (wide ? -1 : where);
        const std::vector<int>& cand = chosen.cand;
        const double ready = chosen.ready;
        int best_p = chosen.p, best_subs = chosen.subs;
        double best_finish = chosen.finish;
        auto ready_without = [&](int skip) { return ready_at(out.xcd[v], skip); };
        // Alternative for an elementwise task: take over the partition and the workgroups of
        // an E' parent with the same output shape on the same XCD. Tile i then depends only on
        // what the same workgroup wrote a moment ago, and the wait for that parent is dropped.
        int follow = -1, follow_kid = KID_NONE;
        long follow_ntiles = 0;
        double follow_finish = 1e300;
        if (allow_local && !wide && !g->resident_all_far) {
            for (int u : parents[v]) {
                if (!g->tasks[u].fn || out.xcd[u] != out.xcd[v] || !(g->nodes[u].out == g->nodes[v].out)) continue;
                if (std::find(g->nodes[v].preds.begin(), g->nodes[v].preds.end(), u) == g->nodes[v].preds.end()) continue;
                long nt = 0;
                const int kid = variant_for(g, v, partition_of(out.kid[u]), &nt);
                if (kid == KID_NONE || nt != out.ntiles[u]) continue;
                double start = ready_without(u);
                for (int w : wgs[u]) start = std::max(start, free_at[w]);
                const long r = (units_for(nt, out.subs[u]) + (long)wgs[u].size() - 1) / (long)wgs[u].size();
                const double f = start + kLocalUs + r * round_us(v, kid, out.subs[u]) + kSyncNearUs;
                if (f < follow_finish) follow_finish = f, follow = u, follow_kid = kid, follow_ntiles = nt;
            }
        }
        long r;
        double begin;
        if (follow >= 0 && follow_finish <= best_finish + 1e-9) {
            out.local_parent[v] = follow;
            out.kid[v] = follow_kid;
            out.ntiles[v] = follow_ntiles;
            out.subs[v] = out.subs[follow];
            wgs[v] = wgs[follow];
            best_finish = follow_finish;
            r = (units_for(follow_ntiles, out.subs[v]) + (long)wgs[v].size() - 1) / (long)wgs[v].size();
            begin = follow_finish - kSyncNearUs - r * round_us(v, follow_kid, out.subs[v]);
        } else {
            out.subs[v] = best_subs;
            wgs[v].assign(cand.begin(), cand.begin() + best_p);
            r = (units_for(ntiles0, best_subs) + best_p - 1) / best_p;
            begin = -1;
        }
        const int p = (int)wgs[v].size();
        const double run = r * round_us(v, out.kid[v], out.subs[v]);
        out.parts[v] = (unsigned)p;
        out.model_run[v] = run;
        // a task spread over several XCDs collects its completions per XCD first
        int peers[8] = {0, 0, 0, 0, 0, 0, 0, 0}, xcds_used = 0;
        for (int j = 0; j < p; ++j) ++peers[wgs[v][j] % 8];
        for (int x = 0; x < 8; ++x) xcds_used += peers[x] > 0;
        const bool two_level = xcds_used > 1 && !knob("NG_NO_TWO_LEVEL");
        out.signals[v] = two_level ? (unsigned)xcds_used : (unsigned)p;
        for (int j = 0; j < p; ++j) {
            const int w = wgs[v][j];
            out.lists[w].push_back(DevEntry{v, j, p, out.subs[v], two_level ? peers[w % 8] : 0});
            free_at[w] = (begin >= 0 ? begin : std::max(ready, free_at[w])) + run + kPublishUs;
        }
        finish[v] = best_finish;
        out.makespan = std::max(out.makespan, best_finish);
        if (debug)
            fprintf(stderr, "PLAN nx=%d v=%d kid=%d ntiles=%ld p=%d r=%ld xcd=%d ready=%.2f cost=%.2f finish=%.2f stream=%d local=%d subs=%d\n",
                    nx, v, out.kid[v], out.ntiles[v], p, r, out.xcd[v], ready, run / r, best_finish, sc.stream_of[v], out.local_parent[v], out.subs[v]);
        for (int c : children[v])
            if (--waiting[c] == 0) open.push(Key(ready_time(c), -tail[c], c));
    }
}

}  // namespace

const PlanKnobs& plan_setting(int k) {
    // far hand-over, spread penalty, 4-outputs-per-thread threshold, near hand-over, publish, far-run factor
    static const PlanKnobs kSettings[kPlanSettings] = {
        PlanKnobs(),                        // the default
        {1.0, 2.0, 3, 0.4, 1.5, 1.2},       // cheaper hand-overs, workgroups busy for longer after a task
        {1.0, 2.0, 3, 0.7, 2.5, 1.2},       // ... much longer: tasks of one stream alternate between workgroups
        {1.0, 2.0, 3, 0.7, 0.6, 1.2},       // ... shorter: a stream stays on few workgroups
        {1.0, 1.0, 3, 0.7, 1.5, 1.2},       // spreads over all XCDs more readily
        {1.0, 2.0, 3, 0.7, 1.5, 1.0},       // far operands cost a tile nothing
        {1.0, 2.0, 1 << 20, 0.7, 1.2, 1.2}, // windowed tasks never take 4 outputs per thread
        {2.0, 2.0, 3, 0.7, 1.2, 1.2},       // a hand-over between XCDs costs twice as much: streams keep to themselves
    };
    return kSettings[std::min(std::max(k, 0), kPlanSettings - 1)];
}

int plan_resident(const ng_graph* g, int n_wg, int xcds, const PlanKnobs& knobs, ResidentPlan& plan) {
    const Schedule& sc = g->sched;
    const int n = (int)g->nodes.size();
    Sim best;
    int best_nx = 0;
    for (int nx : {1, 2, 3, 4, 5, 6, 7, 8}) {
        if (xcds > 0 && nx != xcds) continue;
        Sim s;
        simulate(g, n_wg, nx, knobs, s);
        if (best_nx == 0 || s.makespan < best.makespan) best = std::move(s), best_nx = nx;
    }
    plan.n_wg = n_wg;
    plan.xcds = best_nx;
    plan.est_us = best.makespan;
    plan.order = best.order;
    plan.fused_into = best.fused_into;
    plan.elided = best.elided;
    plan.model_run_us = best.model_run;

    plan.tasks.assign(n, DevTask());
    for (int v = 0; v < n; ++v) {
        DevTask& d = plan.tasks[v];
        std::memset(&d, 0, sizeof d);
        const Task& t = g->tasks[v];
        if (!t.fn) continue;
        d.kid = best.kid[v];
        d.ntiles = (int)best.ntiles[v];
        static_assert(sizeof d.args <= sizeof t.args, "argument blocks");
        std::memcpy(d.args, t.args, sizeof d.args);
    }
    // A tensor crosses XCDs when a direct reader (any edge of E, not only E') runs elsewhere.
    for (int v = 0; v < n; ++v) {
        if (!g->tasks[v].fn) continue;
        const std::vector<int>& preds = g->nodes[v].preds;
        for (size_t j = 0; j < preds.size(); ++j) {
            const int u = preds[j];
            if (!g->tasks[u].fn) continue;          // network input: written before the launch
            const bool far = best.xcd[u] < 0 || best.xcd[v] < 0 || best.xcd[u] != best.xcd[v] || g->resident_all_far;
            if (far) plan.tasks[v].far_in |= 1u << j;
        }
        if (plan.tasks[v].far_in)                    // one far operand: every operand comes through the memory side
            for (int u : preds)
                if (g->tasks[u].fn) plan.tasks[u].release_far = 1;
        if (g->resident_all_far) plan.tasks[v].release_far = 1;
    }
    // the stores into an in-place concat are its producers' stores
    for (int v = n - 1; v >= 0; --v)
        if (best.elided[v] && plan.tasks[v].release_far)
            for (int u : g->nodes[v].preds) plan.tasks[u].release_far = 1;
    // fused pairs: the convolution's argument block gets the batch-norm's coefficients and output
    for (int v = 0; v < n; ++v) {
        const int u = best.fused_into[v];
        if (u < 0) continue;
        const bool c3 = takes_c3_args(best.kid[u]);
        if (g->nodes[v].op == NG_OP_ADD_N) {
            const AddArgs* add = reinterpret_cast<const AddArgs*>(g->tasks[v].args);
            AddEpilogue ea{};
            ea.y = add->y, ea.k = add->k, ea.zpos = -1, ea.far = plan.tasks[v].far_in != 0 ? 1 : 0;
            int q = 0;
            for (int j = 0; j < add->k; ++j) {
                if (g->nodes[v].preds[j] == best.local_parent[v]) ea.zpos = j;
                else if (q < kEpilogueAddMax - 1) ea.x[q++] = add->x[j];
            }
            if (ea.zpos < 0 || q != add->k - 1) return NG_EINVAL;
            if (!has_add_epilogue(best.kid[u])) return NG_EINVAL;
            if (c3) reinterpret_cast<C3AddArgs*>(plan.tasks[u].args)->ea = ea;
            else if (is_pool(best.kid[u])) reinterpret_cast<PoolAddArgs*>(plan.tasks[u].args)->ea = ea;
            else reinterpret_cast<PwAddArgs*>(plan.tasks[u].args)->ea = ea;
        } else {
            const BnArgs* bn = reinterpret_cast<const BnArgs*>(g->tasks[v].args);
            Epilogue ep{bn->scale, bn->shift, bn->y, bn->relu};
            if (c3) reinterpret_cast<C3Args*>(plan.tasks[u].args)->ep = ep;
            else reinterpret_cast<PwArgs*>(plan.tasks[u].args)->ep = ep;
        }
        plan.tasks[u].release_far |= plan.tasks[v].release_far;   // all results of a tile are stored the same way
    }
    // who waits for whom: first what every entry awaits before it starts, then (pass 1) the producers of
    // the other operands of a fused add_n, which its convolution awaits late
    std::vector<std::vector<int>> meg_parents(n);
    for (auto& e : sc.meg)
        if (g->tasks[e.first].fn && g->tasks[e.second].fn) meg_parents[e.second].push_back(e.first);
    // the tasks whose completion stands for the completion of u: u itself, the host it is fused into, or
    // (an in-place concat) what stands for each of its E' parents
    std::function<void(int, std::vector<int>&)> producers_of = [&](int u, std::vector<int>& list) {
        if (best.elided[u]) {
            for (int p : meg_parents[u]) producers_of(p, list);
            return;
        }
        const int src = best.fused_into[u] >= 0 ? best.fused_into[u] : u;
        if (std::find(list.begin(), list.end(), src) == list.end()) list.push_back(src);
    };
    for (int pass = 0; pass < 2; ++pass)
        for (auto& e : sc.meg) {
            if (!g->tasks[e.first].fn || !g->tasks[e.second].fn) continue;
            if (best.local_parent[e.second] == e.first || best.elided[e.second]) continue;   // handed over inside the workgroups / nothing to wait for
            const int dst = best.fused_into[e.second] >= 0 ? best.fused_into[e.second] : e.second; // whose entries wait for it
            if ((dst != e.second) != (pass == 1)) continue;
            std::vector<int> sources;
            producers_of(e.first, sources);
            DevTask& d = plan.tasks[dst];
            for (int src : sources) {
                if (src == dst || std::find(d.parent, d.parent + d.n_parents, src) != d.parent + d.n_parents) continue;
                if (d.n_parents >= NG_MAX_PREDS) return NG_EINVAL;
                d.parent[d.n_parents] = src;
                d.need[d.n_parents] = best.signals[src];
                // producer and consumer on the same single XCD: the completion is signalled through that XCD's L2
                const bool near = best.xcd[src] >= 0 && best.xcd[src] == best.xcd[dst] && !g->resident_all_far &&
                                  !knob("NG_NO_NEAR_COUNTERS");
                if (near) plan.tasks[src].publish |= 1u;
                else plan.tasks[src].publish |= 2u, d.parent_far |= 1u << d.n_parents;
                if (!near && best.signals[src] != best.parts[src]) plan.tasks[src].publish |= 4u;
                ++d.n_parents;
                if (pass == 1) ++d.n_late;
            }
        }
    plan.entries.clear();
    plan.wg_first.assign(n_wg + 1, 0);
    for (int w = 0; w < n_wg; ++w) {
        plan.wg_first[w] = (int)plan.entries.size();
        plan.entries.insert(plan.entries.end(), best.lists[w].begin(), best.lists[w].end());
    }
    plan.wg_first[n_wg] = (int)plan.entries.size();
    return NG_OK;
}

}  // namespace ng

namespace ng {

// Self-check of a device-resident plan against the graph it was made for; true if it holds.
bool resident_plan_is_consistent(const ng_graph* g, const ResidentPlan& plan) {
    // invariants: every tile of every task is covered exactly once, lists ascend in task id,
    // the completions a consumer expects equal the workgroups its producer was split over,
    // and an E' parent that is not waited for has the same tiles on the same workgroups
    bool ok = true;
    const size_t n = g->nodes.size();
    std::vector<std::vector<int>> hits(n);
    std::vector<unsigned> parts(n, 0);
    std::vector<std::vector<long>> where(n);              // (workgroup, first unit, step, subs) per task
    std::vector<int> subs_of(n, 0);
    for (const DevEntry& en : plan.entries) {
        ok = ok && en.subs >= 1 && en.subs <= kSubs && (subs_of[en.task] == 0 || subs_of[en.task] == en.subs);
        subs_of[en.task] = std::min(std::max(en.subs, 1), kSubs);
    }
    auto units_of = [&](int v) { return ((long)plan.tasks[v].ntiles + subs_of[v] - 1) / std::max(subs_of[v], 1); };
    // every list follows one common order of the tasks in which parents come first
    std::vector<int> pos(n, -1);
    for (size_t i = 0; i < plan.order.size(); ++i) {
        const int v = plan.order[i];
        ok = ok && v >= 0 && v < (int)n && g->tasks[v].fn && pos[v] < 0;
        if (v >= 0 && v < (int)n) pos[v] = (int)i;
    }
    for (size_t v = 0; v < n; ++v) ok = ok && ((pos[v] >= 0) == (g->tasks[v].fn != nullptr));
    for (auto& e : g->sched.meg)
        if (g->tasks[e.first].fn && g->tasks[e.second].fn) ok = ok && pos[e.first] < pos[e.second];
    for (int w = 0; w < plan.n_wg && ok; ++w) {
        int last = -1;
        for (int e = plan.wg_first[w]; e < plan.wg_first[w + 1]; ++e) {
            const DevEntry& en = plan.entries[e];
            ok = ok && pos[en.task] > last && en.tile_step > 0 && en.tile_begin >= 0 && en.tile_begin < en.tile_step &&
                 en.tile_begin < units_of(en.task);       // at least one round of tiles: the entry's wait is inside its tile function
            last = pos[en.task];
            ++parts[en.task];
            where[en.task].insert(where[en.task].end(), {(long)w, (long)en.tile_begin, (long)en.tile_step, (long)en.subs});
            if (hits[en.task].empty()) hits[en.task].assign((size_t)units_of(en.task), 0);
            for (long t = en.tile_begin; t < units_of(en.task); t += en.tile_step) ++hits[en.task][(size_t)t];
        }
    }
    // increments of the device-scope counter a waiter may expect: one per participant, or with
    // two-level completion one per XCD on which the task has participants
    std::vector<unsigned> signals(n, 0);
    {
        std::vector<std::vector<int>> on_xcd(n, std::vector<int>(8, 0));
        for (int w = 0; w < plan.n_wg; ++w)
            for (int e = plan.wg_first[w]; e < plan.wg_first[w + 1]; ++e) ++on_xcd[plan.entries[e].task][w % 8];
        for (int w = 0; w < plan.n_wg; ++w)
            for (int e = plan.wg_first[w]; e < plan.wg_first[w + 1]; ++e) {
                const DevEntry& en = plan.entries[e];
                const bool two_level = (plan.tasks[en.task].publish & 4u) != 0;
                ok = ok && (en.xcd_peers == 0 || en.xcd_peers == on_xcd[en.task][w % 8]) && (!two_level || en.xcd_peers > 0);
            }
        for (size_t v = 0; v < n; ++v) {
            int used = 0;
            for (int x = 0; x < 8; ++x) used += on_xcd[v][x] > 0;
            signals[v] = (plan.tasks[v].publish & 4u) ? (unsigned)used : parts[v];
        }
    }
    int n_local = 0, n_fused = 0, n_elided = 0;
    std::vector<int> fused_bns(n, 0), fused_adds(n, 0);
    for (size_t v = 0; v < n; ++v) {
        if (!g->tasks[v].fn) continue;
        if (plan.elided[v]) {
            // an in-place concat: every input lives inside its result, no entries, no waits
            ++n_elided;
            ok = ok && g->nodes[v].op == NG_OP_CONCAT && hits[v].empty() && plan.tasks[v].n_parents == 0 && plan.fused_into[v] < 0;
            for (int u : g->nodes[v].preds) ok = ok && g->alias_of[u] == (int)v && pos[u] < pos[v];
            continue;
        }
        const int host = plan.fused_into[v];
        if (host >= 0) {
            // a fused task has no entries and no waits of its own; its convolution covers the same tile
            // grid, comes earlier in the order and carries its coefficients / operands and output address
            ++n_fused;
            const int hk = plan.tasks[host].kid;
            const bool c3 = takes_c3_args(hk), pool = is_pool(hk), pw = !c3 && !pool && has_bn_epilogue(hk);
            static const Epilogue none{};
            const Epilogue* ep = c3 ? &reinterpret_cast<const C3Args*>(plan.tasks[host].args)->ep
                                    : pw ? &reinterpret_cast<const PwArgs*>(plan.tasks[host].args)->ep : &none;
            const AddEpilogue* ea = c3 ? &reinterpret_cast<const C3AddArgs*>(plan.tasks[host].args)->ea
                                       : pool ? &reinterpret_cast<const PoolAddArgs*>(plan.tasks[host].args)->ea
                                              : &reinterpret_cast<const PwAddArgs*>(plan.tasks[host].args)->ea;
            const bool is_add = g->nodes[v].op == NG_OP_ADD_N;
            ok = ok && (is_add ? add_variant(plain_variant(hk)) != KID_NONE : has_bn_epilogue(hk)) && hits[v].empty() &&
                 plan.tasks[v].n_parents == 0 && plan.fused_into[host] < 0 && pos[host] < pos[v] &&
                 g->nodes[host].out == g->nodes[v].out && (plan.tasks[host].release_far || !plan.tasks[v].release_far) &&
                 (!is_add || (partition_of(hk) == partition_of(plan.tasks[v].kid) && plan.tasks[host].ntiles == plan.tasks[v].ntiles));
            if (g->nodes[v].op == NG_OP_ADD_N) {
                ok = ok && has_add_epilogue(hk);
                const AddArgs* add = reinterpret_cast<const AddArgs*>(plan.tasks[v].args);
                const float* held = ep->y != nullptr ? ep->y
                                    : c3 ? reinterpret_cast<const C3Args*>(plan.tasks[host].args)->y
                                         : pool ? reinterpret_cast<const PoolArgs*>(plan.tasks[host].args)->y
                                                : reinterpret_cast<const PwArgs*>(plan.tasks[host].args)->y;
                ok = ok && ea->y == add->y && ea->k == add->k && add->k >= 2 && add->k <= kEpilogueAddMax && ea->zpos >= 0 &&
                     ea->zpos < add->k && (ea->far != 0) == (plan.tasks[v].far_in != 0);
                int q = 0, late = 0;
                for (int j = 0; j < add->k && ok; ++j) {
                    if (j == ea->zpos) ok = add->x[j] == held;
                    else ok = ea->x[q++] == add->x[j];
                }
                // every E' parent of the add_n other than the fused operand is awaited late by the convolution
                for (auto& e : g->sched.meg)
                    if (e.second == (int)v && g->tasks[e.first].fn) {
                        const int src = plan.fused_into[e.first] >= 0 ? plan.fused_into[e.first] : e.first;
                        if (src == host) continue;
                        ++late;
                        const DevTask& h = plan.tasks[host];
                        ok = ok && !plan.elided[src] && std::find(h.parent, h.parent + h.n_parents, src) != h.parent + h.n_parents;
                    }
                ok = ok && late >= (int)plan.tasks[host].n_late;
                ++fused_adds[host];
            } else {
                const BnArgs* bn = reinterpret_cast<const BnArgs*>(plan.tasks[v].args);
                ok = ok && g->nodes[v].preds.size() == 1 && g->nodes[v].preds[0] == host && ep->y == bn->y &&
                     ep->scale == bn->scale && ep->shift == bn->shift && ep->relu == bn->relu;
                ++fused_bns[host];
            }
            continue;
        }
        ok = ok && plan.tasks[v].ntiles > 0 && hits[v].size() == (size_t)units_of((int)v);
        for (int h : hits[v]) ok = ok && h == 1;
        const DevTask& d = plan.tasks[v];
        for (int j = 0; j < d.n_parents; ++j) ok = ok && pos[d.parent[j]] < pos[v] && d.need[j] == signals[d.parent[j]] && parts[d.parent[j]] > 0;
    }
    for (auto& e : g->sched.meg) {
        const int u = e.first, v = e.second;
        if (!g->tasks[u].fn || !g->tasks[v].fn) continue;
        if (plan.elided[v]) continue;                                              // waits for nothing
        const int dst = plan.fused_into[v] >= 0 ? plan.fused_into[v] : v;         // whose workgroups wait for it
        const DevTask& d = plan.tasks[dst];
        // whose workgroups store u's result: u, its host, or (in-place concat) those of its E' parents
        std::vector<int> sources;
        std::function<void(int)> expand = [&](int t) {
            if (plan.elided[t]) {
                for (auto& f : g->sched.meg)
                    if (f.second == t && g->tasks[f.first].fn) expand(f.first);
            } else {
                sources.push_back(plan.fused_into[t] >= 0 ? plan.fused_into[t] : t);
            }
        };
        expand(u);
        for (int src : sources) {
            if (src == dst) continue;                                             // fused pair, checked above
            if (std::find(d.parent, d.parent + d.n_parents, src) != d.parent + d.n_parents) continue;
            ++n_local;
            const int part = partition_of(plan.tasks[u].kid);
            ok = ok && !plan.elided[u] && plan.fused_into[v] < 0 && part != PART_NONE && part == partition_of(d.kid) &&
                 plan.tasks[u].ntiles == d.ntiles && g->nodes[u].out == g->nodes[v].out && where[src] == where[v];
        }
    }
    // epilogues are there exactly where a task was fused; late parents only with a fused add_n
    for (size_t u = 0; u < n; ++u) {
        const int k = plan.tasks[u].kid;
        if (!g->tasks[u].fn) continue;
        const bool c3 = takes_c3_args(k), pw = !c3 && has_bn_epilogue(k);
        ok = ok && fused_bns[u] <= 1 && fused_adds[u] <= 1 && (c3 || pw || fused_bns[u] == 0) && (add_variant(plain_variant(k)) != KID_NONE || fused_adds[u] == 0) &&
             (fused_adds[u] == 1 || plan.tasks[u].n_late == 0) && plan.tasks[u].n_late <= (unsigned)plan.tasks[u].n_parents;
        ok = ok && has_add_epilogue(k) == (fused_adds[u] == 1);
        if (c3) ok = ok && (reinterpret_cast<const C3Args*>(plan.tasks[u].args)->ep.y != nullptr) == (fused_bns[u] == 1);
        if (pw) ok = ok && (reinterpret_cast<const PwArgs*>(plan.tasks[u].args)->ep.y != nullptr) == (fused_bns[u] == 1);
    }
    if (knob("NG_PLAN_DEBUG")) fprintf(stderr, "PLAN local hand-overs: %d, fused: %d, concats in place: %d, self-check %s\n", n_local, n_fused, n_elided, ok ? "passed" : "FAILED");
    return ok;
}

}  // namespace ng

extern "C" int ng_resident_dry_plan(ng_graph* g, int n_workgroups, int xcds, double* expected_us, int* n_entries,
                                    int* n_far_edges, int* coverage_ok) {
    return ng_resident_dry_plan_setting(g, 0, n_workgroups, xcds, expected_us, n_entries, n_far_edges, coverage_ok);
}

extern "C" int ng_resident_dry_plan_setting(ng_graph* g, int setting, int n_workgroups, int xcds, double* expected_us,
                                            int* n_entries, int* n_far_edges, int* coverage_ok) {
    using namespace ng;
    if (!g) return NG_EINVAL;
    if (g->phase < PLANNED) return g->fail(NG_ESTATE, "ng_resident_dry_plan: call ng_plan_memory first");
    if (n_workgroups < 8 || n_workgroups % 8 != 0 || xcds < 0 || xcds > 8)
        return g->fail(NG_EINVAL, "ng_resident_dry_plan: workgroups must be a positive multiple of 8, xcds 0..8");
    if (setting < 0 || setting >= kPlanSettings)
        return g->fail(NG_EINVAL, "ng_resident_dry_plan_setting: setting must be 0..%d", kPlanSettings - 1);
    std::vector<Task> saved;
    saved.swap(g->tasks);
    g->dry_run = true;
    g->tasks.assign(g->nodes.size(), Task());
    int rc = NG_OK;
    char* fake_arena = reinterpret_cast<char*>(0x100000000ull);
    static float fake_constants;
    for (int v = 0; v < (int)g->nodes.size() && rc == NG_OK; ++v) rc = build_task(g, v, fake_arena, &fake_constants, g->tasks[v]);
    ResidentPlan plan;
    if (rc == NG_OK && plan_resident(g, n_workgroups, xcds, plan_setting(setting), plan) != NG_OK) rc = g->fail(NG_EINVAL, "too many E' parents");
    if (rc == NG_OK) {
        if (expected_us) *expected_us = plan.est_us;
        if (n_entries) *n_entries = (int)plan.entries.size();
        int far = 0;
        for (auto& t : plan.tasks) far += __builtin_popcount(t.far_in);
        if (n_far_edges) *n_far_edges = far;
        const bool ok = resident_plan_is_consistent(g, plan);
        if (coverage_ok) *coverage_ok = ok;
    }
    g->dry_run = false;
    g->tasks.swap(saved);
    return rc;
}
