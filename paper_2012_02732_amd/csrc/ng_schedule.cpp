// Stream assignment and synchronisation plan: Algorithm 1 of the Nimble paper
// (arXiv 2012.02732, Section 4.2) and the synchronisation model of its Appendix A.
//
//   Step 1    G' = minimum equivalent graph of G (unique for a DAG).
//   Step 2-3  maximum matching of the bipartite graph whose edges are E'.
//   Step 4-5  nodes joined by matched edges share a stream ("chains").
//   Lambda    an E' edge is the only path between its ends (Lemma 1), so it needs its own
//             synchronisation exactly when its ends sit on different streams; the count is
//             |E'| - |M| for Algorithm 1's assignment (Theorem 3) and |E'| - |Q(f)| for any
//             assignment with maximum logical concurrency (Lemma 4).
//
// Choices the paper leaves open, fixed here so that the result is reproducible:
//   * the matching is found by augmenting paths, left nodes in ascending id, candidate
//     right nodes in ascending id;
//   * Step 2 on E' alone yields a minimum path cover of G', which can use more streams
//     than the widest antichain. The E' matching is kept as it is and chains are then
//     joined tail to head wherever the head is reachable from the tail (this neither adds
//     nor removes a same-stream E' edge, so the synchronisation count is unchanged). A
//     last augmenting pass over the full closure, which may re-route earlier pairs and is
//     normally idle, guarantees stream count = antichain width (Dilworth);
//   * streams are numbered by the smallest node id they hold; tasks are submitted in
//     ascending id; a producer with cross-stream E' successors records one event, each such
//     successor waits for it before launching.
#include <algorithm>
#include <limits>
#include <cstdint>

#include "ng_internal.h"

namespace ng {
namespace {

// Row-major bit matrix.
struct BitMatrix {
    int n = 0, words = 0;
    std::vector<uint64_t> bits;
    explicit BitMatrix(int n_) : n(n_), words((n_ + 63) / 64), bits((size_t)n_ * ((n_ + 63) / 64), 0) {}
    uint64_t* row(int r) { return bits.data() + (size_t)r * words; }
    const uint64_t* row(int r) const { return bits.data() + (size_t)r * words; }
    void set(int r, int c) { row(r)[c >> 6] |= 1ull << (c & 63); }
    bool get(int r, int c) const { return row(r)[c >> 6] >> (c & 63) & 1; }
};

// Bipartite matching by augmenting paths with an explicit stack. `adj[x]` lists the
// candidate right nodes of left node x in the order they are tried.
struct Matcher {
    const std::vector<std::vector<int>>& adj;
    std::vector<int>&left_to, &right_to;
    std::vector<int> stamp, cursor;
    int round = 0;

    Matcher(const std::vector<std::vector<int>>& a, std::vector<int>& l, std::vector<int>& r)
        : adj(a), left_to(l), right_to(r), stamp(l.size(), 0), cursor(l.size(), 0) {}

    bool augment_from(int root) {
        ++round;
        std::vector<int> path_x{root}, path_y;     // path_y[i] = right node chosen at path_x[i]
        cursor[root] = 0;
        while (!path_x.empty()) {
            const int x = path_x.back();
            bool descended = false;
            while (cursor[x] < (int)adj[x].size()) {
                const int y = adj[x][cursor[x]++];
                if (stamp[y] == round) continue;
                stamp[y] = round;
                if (right_to[y] < 0) {             // free right node: flip the whole path
                    path_y.push_back(y);
                    for (size_t i = 0; i < path_x.size(); ++i) {
                        left_to[path_x[i]] = path_y[i];
                        right_to[path_y[i]] = path_x[i];
                    }
                    return true;
                }
                path_y.push_back(y);               // try to move y's partner elsewhere
                path_x.push_back(right_to[y]);
                cursor[right_to[y]] = 0;
                descended = true;
                break;
            }
            if (!descended) {
                path_x.pop_back();
                if (!path_y.empty()) path_y.pop_back();   // also forget the edge that led to x
            }
        }
        return false;
    }

    void run(const std::vector<int>& lefts) {
        for (int x : lefts)
            if (left_to[x] < 0) augment_from(x);
    }
};

}  // namespace

namespace {

// Minimum-cost perfect assignment of an n x n integer cost matrix (row-major), O(n^3): the
// classic potential method - rows are added one at a time, each by a shortest augmenting path
// over reduced costs. assigned_col[i] = column of row i.
void assign_min_cost(int n, const std::vector<long>& cost, std::vector<int>& assigned_col) {
    const long kInf = std::numeric_limits<long>::max() / 4;
    std::vector<long> pot_row(n + 1, 0), pot_col(n + 1, 0), slack(n + 1);
    std::vector<int> row_of_col(n + 1, 0), came_from(n + 1, 0);    // 1-based; column 0 is a virtual start
    std::vector<char> used(n + 1);
    for (int i = 1; i <= n; ++i) {
        row_of_col[0] = i;
        int col = 0;
        std::fill(slack.begin(), slack.end(), kInf);
        std::fill(used.begin(), used.end(), 0);
        do {
            used[col] = 1;
            const int row = row_of_col[col];
            long delta = kInf;
            int next_col = 0;
            for (int j = 1; j <= n; ++j) {
                if (used[j]) continue;
                const long reduced = cost[(size_t)(row - 1) * n + (j - 1)] - pot_row[row] - pot_col[j];
                if (reduced < slack[j]) slack[j] = reduced, came_from[j] = col;
                if (slack[j] < delta) delta = slack[j], next_col = j;
            }
            for (int j = 0; j <= n; ++j) {
                if (used[j]) pot_row[row_of_col[j]] += delta, pot_col[j] -= delta;
                else slack[j] -= delta;
            }
            col = next_col;
        } while (row_of_col[col] != 0);
        do {                                                   // flip the path back to the start
            const int before = came_from[col];
            row_of_col[col] = row_of_col[before];
            col = before;
        } while (col != 0);
    }
    assigned_col.assign(n, -1);
    for (int j = 1; j <= n; ++j) assigned_col[row_of_col[j] - 1] = j - 1;
}

}  // namespace

void compute_schedule(int n, const std::vector<std::pair<int, int>>& raw_edges, Schedule& s, bool exact) {
    s = Schedule();
    std::vector<std::pair<int, int>> edges = raw_edges;
    std::sort(edges.begin(), edges.end());
    edges.erase(std::unique(edges.begin(), edges.end()), edges.end());

    // Descendants (reach) by a reverse sweep; ancestors (anc) by transposition.
    BitMatrix reach(n), anc(n);
    std::vector<std::vector<int>> succ(n);
    for (auto& e : edges) succ[e.first].push_back(e.second);
    for (int u = n - 1; u >= 0; --u)
        for (int v : succ[u]) {
            reach.set(u, v);
            uint64_t* a = reach.row(u);
            const uint64_t* b = reach.row(v);
            for (int w = 0; w < reach.words; ++w) a[w] |= b[w];
        }
    for (int u = 0; u < n; ++u)
        for (int v = u + 1; v < n; ++v)
            if (reach.get(u, v)) anc.set(v, u);

    s.solo.assign(n, 0);
    for (int v = 0; v < n; ++v) {
        int comparable = 0;
        for (int w = 0; w < reach.words; ++w)
            comparable += __builtin_popcountll(reach.row(v)[w]) + __builtin_popcountll(anc.row(v)[w]);
        s.solo[v] = comparable == n - 1;
    }

    // Step 1: (u, v) stays iff no node lies strictly between u and v.
    for (auto& e : edges) {
        const uint64_t* a = reach.row(e.first);
        const uint64_t* b = anc.row(e.second);
        bool between = false;
        for (int w = 0; w < reach.words && !between; ++w) between = (a[w] & b[w]) != 0;
        if (!between) s.meg.push_back(e);
    }

    // Steps 2-3 on E'.
    std::vector<std::vector<int>> adj(n);
    for (auto& e : s.meg) adj[e.first].push_back(e.second);
    std::vector<int> next(n, -1), prev(n, -1), all(n);
    for (int v = 0; v < n; ++v) all[v] = v;
    {
        Matcher m(adj, next, prev);
        m.run(all);
    }
    for (int v = 0; v < n; ++v) s.n_matching += next[v] >= 0;

    auto label_paths = [&](std::vector<int>& label) {
        label.assign(n, -1);
        int count = 0;
        for (int v = 0; v < n; ++v) {
            if (label[v] >= 0) continue;
            for (int w = v; w >= 0; w = next[w]) label[w] = count;
            ++count;
        }
        return count;
    };
    // Steps 4-5: the merged sets are exactly the paths of the matching.
    s.n_chains = label_paths(s.chain_of);

    if (exact) {
        // Streams = a partition into the fewest chains of the closure (the widest antichain, Dilworth) that,
        // among those, keeps the most E' edges inside a stream, i.e. needs the fewest synchronisations
        // (a same-stream E' edge is always a pair of neighbours on its chain, so it is a matched pair):
        // a maximum matching of the closure's bipartite graph with as many E' edges as possible. As an
        // assignment problem: a closure pair costs -(n + 1), an E' pair one less, anything else 0, so one
        // more matched pair always outweighs any number of E' pairs.
        std::vector<long> cost((size_t)n * n, 0);
        for (int u = 0; u < n; ++u)
            for (int v = u + 1; v < n; ++v)
                if (reach.get(u, v)) cost[(size_t)u * n + v] = -(long)(n + 1);
        for (auto& e : s.meg) cost[(size_t)e.first * n + e.second] -= 1;
        std::vector<int> col;
        assign_min_cost(n, cost, col);
        std::fill(next.begin(), next.end(), -1);
        std::fill(prev.begin(), prev.end(), -1);
        for (int u = 0; u < n; ++u)
            if (col[u] > u && reach.get(u, col[u])) next[u] = col[u], prev[col[u]] = u;
    } else {
    // Join chains: tails (no successor in the matching) to reachable heads (no predecessor).
    {
        std::vector<int> tails;
        std::vector<std::vector<int>> adj2(n);
        for (int t = 0; t < n; ++t) {
            if (next[t] >= 0) continue;
            tails.push_back(t);
            for (int h = t + 1; h < n; ++h)
                if (prev[h] < 0 && reach.get(t, h)) adj2[t].push_back(h);
        }
        Matcher m(adj2, next, prev);
        m.run(tails);
    }
    // Guarantee the antichain width: augment over the whole closure, E' successors first.
    {
        std::vector<std::vector<int>> adj3(n);
        for (int u = 0; u < n; ++u) {
            adj3[u] = adj[u];
            for (int v = u + 1; v < n; ++v)
                if (reach.get(u, v) && !std::binary_search(adj[u].begin(), adj[u].end(), v)) adj3[u].push_back(v);
        }
        Matcher m(adj3, next, prev);
        m.run(all);
    }
    }
    s.n_streams = label_paths(s.stream_of);

    // Synchronisation plan and events.
    s.event_of.assign(n, -1);
    s.waits.assign(n, {});
    for (auto& e : s.meg)
        if (s.stream_of[e.first] != s.stream_of[e.second]) {
            s.sync.push_back(e);
            s.event_of[e.first] = 0;
        }
    for (int v = 0; v < n; ++v)
        if (s.event_of[v] == 0) s.event_of[v] = s.n_events++;
    for (auto& e : s.sync) s.waits[e.second].push_back(e.first);   // sync is sorted by producer

    s.order.resize(n);
    for (int v = 0; v < n; ++v) s.order[v] = v;

    // Capture scaffolding.
    std::vector<int> first(s.n_streams, -1);
    for (int v = n - 1; v >= 0; --v) first[s.stream_of[v]] = v;
    for (int st = 1; st < s.n_streams; ++st) {
        if (s.waits[first[st]].empty()) s.fork.push_back(st);
        s.join.push_back(st);
    }
}

}  // namespace ng
