// Registration, shape inference, static memory plan and host-side queries.
// Paper: Nimble (arXiv 2012.02732), Section 4 (input is a static operator DAG with a
// fixed input shape) and Section 4.1 (all shapes and all memory are fixed ahead of time).
#include <algorithm>
#include <cstdlib>
#include <cstring>
#include <new>

#include "ng_internal.h"

using namespace ng;

namespace {

int conv_out(int64_t size, int k, int stride, int pad) {
    return (int)((size + 2 * pad - k) / stride + 1);
}

bool in_set(int v, int a, int b) { return v == a || v == b; }

// Output shape of an operator, or an error text. Mirrors the operator table in the header.
const char* infer_shape(const ng_graph* g, int op, ng_op_params& p, const int* preds, int n_preds,
                        int n_weights, Shape& out, int& code) {
    code = NG_EINVAL;
    auto in = [&](int j) -> const Shape& { return g->nodes[preds[j]].out; };
    auto need = [&](int np, int nw) { return n_preds == np && n_weights == nw; };
    switch (op) {
        case NG_OP_CONV1X1:
            if (!need(1, 1)) return "conv1x1 takes 1 input and 1 weight";
            if (p.cout <= 0) return "conv1x1: cout must be positive";
            out = in(0);
            out.c = p.cout;
            return nullptr;
        case NG_OP_DWCONV: {
            if (!need(1, 1)) return "dwconv takes 1 input and 1 weight";
            if (!in_set(p.k, 3, 5) || !in_set(p.stride, 1, 2)) return "dwconv: k in {3,5}, stride in {1,2}";
            out = in(0);
            out.h = conv_out(in(0).h, p.k, p.stride, p.k / 2);
            out.w = conv_out(in(0).w, p.k, p.stride, p.k / 2);
            break;
        }
        case NG_OP_CONV3X3:
            if (!need(1, 1)) return "conv3x3 takes 1 input and 1 weight";
            if (p.cout <= 0 || !in_set(p.stride, 1, 2) || !in_set(p.pad, 0, 1))
                return "conv3x3: cout > 0, stride in {1,2}, pad in {0,1}";
            out = in(0);
            out.c = p.cout;
            out.h = conv_out(in(0).h, 3, p.stride, p.pad);
            out.w = conv_out(in(0).w, 3, p.stride, p.pad);
            break;
        case NG_OP_BN_ACT:
            if (!need(1, 4)) return "bn_act takes 1 input and 4 weights";
            if (!(p.eps >= 0.f)) return "bn_act: eps must be >= 0";
            out = in(0);
            return nullptr;
        case NG_OP_RELU:
            if (!need(1, 0)) return "relu takes 1 input and no weights";
            out = in(0);
            return nullptr;
        case NG_OP_ADD_N:
            if (n_preds < 2 || n_preds > NG_MAX_PREDS || n_weights != 0) return "add_n takes 2..8 inputs";
            for (int j = 1; j < n_preds; ++j)
                if (!(in(j) == in(0))) {
                    code = NG_ESHAPE;
                    return "add_n: inputs differ in shape";
                }
            out = in(0);
            return nullptr;
        case NG_OP_CONCAT: {
            if (n_preds < 1 || n_preds > NG_MAX_PREDS || n_weights != 0) return "concat takes 1..8 inputs";
            out = in(0);
            out.c = 0;
            for (int j = 0; j < n_preds; ++j) {
                if (p.slice_hi[j] == 0) {
                    p.slice_lo[j] = 0;
                    p.slice_hi[j] = (int32_t)in(j).c;
                }
                if (in(j).n != in(0).n || in(j).h != in(0).h || in(j).w != in(0).w) {
                    code = NG_ESHAPE;
                    return "concat: inputs differ in n, h or w";
                }
                if (p.slice_lo[j] < 0 || p.slice_lo[j] >= p.slice_hi[j] || p.slice_hi[j] > in(j).c) {
                    code = NG_ESHAPE;
                    return "concat: channel slice out of range";
                }
                out.c += p.slice_hi[j] - p.slice_lo[j];
            }
            return nullptr;
        }
        case NG_OP_POOL:
            if (!need(1, 0)) return "pool takes 1 input and no weights";
            if (!in_set(p.pool_mode, 0, 1) || !in_set(p.stride, 1, 2) || !in_set(p.pad, 0, 1))
                return "pool: mode in {0,1}, stride in {1,2}, pad in {0,1}";
            out = in(0);
            out.h = conv_out(in(0).h, 3, p.stride, p.pad);
            out.w = conv_out(in(0).w, 3, p.stride, p.pad);
            break;
        case NG_OP_GLOBAL_AVGPOOL:
            if (!need(1, 0)) return "global_avgpool takes 1 input and no weights";
            out = in(0);
            out.h = out.w = 1;
            return nullptr;
        case NG_OP_FC:
            if (!need(1, 2)) return "fc takes 1 input and 2 weights";
            if (p.cout <= 0) return "fc: cout must be positive";
            if (in(0).h != 1 || in(0).w != 1) {
                code = NG_ESHAPE;
                return "fc: input must be [n][c][1][1]";
            }
            out = in(0);
            out.c = p.cout;
            return nullptr;
        // ---- backward operators: in(0) = dy, in(1) = x, the forward operator's input ----
        case NG_OP_CONV1X1_DGRAD:
            if (!need(1, 1)) return "conv1x1_dgrad takes dy and the forward weights";
            if (p.cout <= 0) return "conv1x1_dgrad: cout (channels of the result) must be positive";
            out = in(0);
            out.c = p.cout;
            return nullptr;
        case NG_OP_CONV1X1_WGRAD:
            if (!need(2, 0)) return "conv1x1_wgrad takes dy and x";
            if (in(0).n != in(1).n || in(0).h != in(1).h || in(0).w != in(1).w) {
                code = NG_ESHAPE;
                return "conv1x1_wgrad: dy and x differ in n, h or w";
            }
            out = Shape{in(0).c, in(1).c, 1, 1};
            return nullptr;
        case NG_OP_CONV3X3_DGRAD:
        case NG_OP_CONV3X3_WGRAD: {
            const bool dgrad = op == NG_OP_CONV3X3_DGRAD;
            if (!need(2, dgrad ? 1 : 0)) return "conv3x3 backward takes dy and x (dgrad: and the forward weights)";
            if (!in_set(p.stride, 1, 2) || !in_set(p.pad, 0, 1)) return "conv3x3 backward: stride in {1,2}, pad in {0,1}";
            if (in(0).n != in(1).n || conv_out(in(1).h, 3, p.stride, p.pad) != in(0).h || conv_out(in(1).w, 3, p.stride, p.pad) != in(0).w) {
                code = NG_ESHAPE;
                return "conv3x3 backward: dy does not have the shape the forward convolution gives for x";
            }
            out = dgrad ? in(1) : Shape{in(0).c, in(1).c, 3, 3};
            return nullptr;
        }
        case NG_OP_DWCONV_DGRAD:
        case NG_OP_DWCONV_WGRAD: {
            const bool dgrad = op == NG_OP_DWCONV_DGRAD;
            if (!need(2, dgrad ? 1 : 0)) return "dwconv backward takes dy and x (dgrad: and the forward weights)";
            if (!in_set(p.k, 3, 5) || !in_set(p.stride, 1, 2)) return "dwconv backward: k in {3,5}, stride in {1,2}";
            if (in(0).n != in(1).n || in(0).c != in(1).c || conv_out(in(1).h, p.k, p.stride, p.k / 2) != in(0).h ||
                conv_out(in(1).w, p.k, p.stride, p.k / 2) != in(0).w) {
                code = NG_ESHAPE;
                return "dwconv backward: dy does not have the shape the forward operator gives for x";
            }
            out = dgrad ? in(1) : Shape{1, in(1).c, p.k, p.k};
            return nullptr;
        }
        case NG_OP_BN_ACT_DGRAD:
        case NG_OP_BN_ACT_WGRAD:
            if (!need(2, 4)) return "bn_act backward takes dy, x and the 4 forward weights";
            if (!(p.eps >= 0.f)) return "bn_act backward: eps must be >= 0";
            if (!(in(0) == in(1))) {
                code = NG_ESHAPE;
                return "bn_act backward: dy and x differ in shape";
            }
            out = op == NG_OP_BN_ACT_DGRAD ? in(1) : Shape{2, in(1).c, 1, 1};
            return nullptr;
        case NG_OP_RELU_DGRAD:
            if (!need(2, 0)) return "relu_dgrad takes dy and x";
            if (!(in(0) == in(1))) {
                code = NG_ESHAPE;
                return "relu_dgrad: dy and x differ in shape";
            }
            out = in(1);
            return nullptr;
        case NG_OP_POOL_DGRAD:
            if (!need(2, 0)) return "pool_dgrad takes dy and x";
            if (!in_set(p.pool_mode, 0, 1) || !in_set(p.stride, 1, 2) || !in_set(p.pad, 0, 1))
                return "pool_dgrad: mode in {0,1}, stride in {1,2}, pad in {0,1}";
            if (in(0).n != in(1).n || in(0).c != in(1).c || conv_out(in(1).h, 3, p.stride, p.pad) != in(0).h ||
                conv_out(in(1).w, 3, p.stride, p.pad) != in(0).w) {
                code = NG_ESHAPE;
                return "pool_dgrad: dy does not have the shape the forward pool gives for x";
            }
            out = in(1);
            return nullptr;
        case NG_OP_GAP_DGRAD:
            if (!need(2, 0)) return "global_avgpool_dgrad takes dy and x";
            if (in(0).n != in(1).n || in(0).c != in(1).c || in(0).h != 1 || in(0).w != 1) {
                code = NG_ESHAPE;
                return "global_avgpool_dgrad: dy must be [n][c][1][1] for x [n][c][h][w]";
            }
            out = in(1);
            return nullptr;
        case NG_OP_CHANNEL_SUM:
            if (!need(1, 0)) return "channel_sum takes 1 input";
            out = Shape{1, in(0).c, 1, 1};
            return nullptr;
        case NG_OP_SLICE_PAD: {
            if (!need(1, 0)) return "slice_pad takes 1 input";
            const int cnt = p.slice_hi[0] - p.slice_lo[0];
            if (p.cout <= 0 || p.slice_lo[0] < 0 || cnt <= 0 || p.slice_hi[0] > in(0).c || p.slice_lo[1] < 0 || p.slice_lo[1] + cnt > p.cout) {
                code = NG_ESHAPE;
                return "slice_pad: channel ranges out of range";
            }
            out = in(0);
            out.c = p.cout;
            return nullptr;
        }
        case NG_OP_SGD_UPDATE:
            if (n_preds < 1 || n_weights != 1) return "sgd_update takes the gradient (and nodes to run after) and 1 weight buffer";
            if (p.cout <= 0 || p.slice_lo[0] < 0 || (int64_t)p.slice_lo[0] + p.cout > in(0).elems()) {
                code = NG_ESHAPE;
                return "sgd_update: [offset, offset + elements) is not inside the gradient tensor";
            }
            if (!(p.lr == p.lr)) return "sgd_update: lr is not a number";
            out = Shape{1, 1, 1, 1};
            return nullptr;
        default:
            return "unknown operator kind";
    }
    if (out.h <= 0 || out.w <= 0) {
        code = NG_ESHAPE;
        return "window does not fit the input";
    }
    return nullptr;
}

}  // namespace

extern "C" {

const char* ng_version(void) { return "nimble_graph 0.1 (gfx950)"; }

int ng_create(ng_graph** out) {
    if (!out) return NG_EINVAL;
    *out = new (std::nothrow) ng_graph();
    return *out ? NG_OK : NG_ENOMEM;
}

void ng_destroy(ng_graph* g) {
    if (!g) return;
    destroy_runtime(g);
    delete g;
}

const char* ng_last_error(const ng_graph* g) { return g ? g->err.c_str() : "null graph"; }

int ng_add_input(ng_graph* g, const int64_t nchw[4], int* id) {
    if (!g) return NG_EINVAL;
    if (!nchw || !id) return g->fail(NG_EINVAL, "ng_add_input: null argument");
    if (g->phase != BUILDING) return g->fail(NG_ESTATE, "ng_add_input: registration is closed");
    for (int i = 0; i < 4; ++i)
        if (nchw[i] <= 0 || nchw[i] > (1 << 24)) return g->fail(NG_ESHAPE, "ng_add_input: bad extent %lld", (long long)nchw[i]);
    Node nd;
    nd.op = NG_OP_INPUT;
    nd.out = Shape{nchw[0], nchw[1], nchw[2], nchw[3]};
    g->nodes.push_back(nd);
    *id = (int)g->nodes.size() - 1;
    return NG_OK;
}

int ng_add_node(ng_graph* g, int op_kind, const ng_op_params* p, const int* preds, int n_preds,
                const void* const* dev_weights, int n_weights, int* id) {
    if (!g) return NG_EINVAL;
    if (!id || n_preds < 0 || n_weights < 0 || (n_preds > 0 && !preds) || (n_weights > 0 && !dev_weights))
        return g->fail(NG_EINVAL, "ng_add_node: null or negative argument");
    if (g->phase != BUILDING) return g->fail(NG_ESTATE, "ng_add_node: registration is closed");
    if (op_kind == NG_OP_INPUT) return g->fail(NG_EINVAL, "ng_add_node: use ng_add_input for inputs");
    if (n_preds == 0 || n_preds > NG_MAX_PREDS) return g->fail(NG_EINVAL, "ng_add_node: needs 1..%d predecessors", NG_MAX_PREDS);
    for (int j = 0; j < n_preds; ++j)
        if (preds[j] < 0 || preds[j] >= (int)g->nodes.size())
            return g->fail(NG_EINVAL, "ng_add_node: predecessor id %d does not exist", preds[j]);
    Node nd;
    nd.op = op_kind;
    if (p) nd.p = *p;
    int code = NG_EINVAL;
    if (const char* msg = infer_shape(g, op_kind, nd.p, preds, n_preds, n_weights, nd.out, code))
        return g->fail(code, "ng_add_node(node %d): %s", (int)g->nodes.size(), msg);
    if (nd.out.elems() <= 0 || nd.out.elems() >= ((int64_t)1 << 31))
        return g->fail(NG_ESHAPE, "ng_add_node: tensor of %lld elements is not supported", (long long)nd.out.elems());
    nd.preds.assign(preds, preds + n_preds);
    nd.weights.assign(dev_weights, dev_weights + n_weights);
    g->nodes.push_back(std::move(nd));
    *id = (int)g->nodes.size() - 1;
    return NG_OK;
}

int ng_mark_output(ng_graph* g, int id) {
    if (!g) return NG_EINVAL;
    if (id < 0 || id >= (int)g->nodes.size()) return g->fail(NG_EINVAL, "ng_mark_output: no node %d", id);
    g->nodes[id].is_output = true;
    return NG_OK;
}

int ng_num_nodes(const ng_graph* g) { return g ? (int)g->nodes.size() : NG_EINVAL; }

int ng_node_shape(const ng_graph* g, int id, int64_t nchw[4]) {
    if (!g || !nchw || id < 0 || id >= (int)g->nodes.size()) return NG_EINVAL;
    const Shape& s = g->nodes[id].out;
    nchw[0] = s.n, nchw[1] = s.c, nchw[2] = s.h, nchw[3] = s.w;
    return NG_OK;
}

int ng_set_assignment(ng_graph* g, int assignment) {
    if (!g) return NG_EINVAL;
    if (g->phase != BUILDING) return g->fail(NG_ESTATE, "ng_set_assignment: already scheduled");
    if (assignment != NG_ASSIGN_ALGORITHM1 && assignment != NG_ASSIGN_EXACT)
        return g->fail(NG_EINVAL, "ng_set_assignment: unknown assignment %d", assignment);
    g->assignment = assignment;
    return NG_OK;
}

int ng_schedule(ng_graph* g) {
    if (!g) return NG_EINVAL;
    if (g->phase != BUILDING) return g->fail(NG_ESTATE, "ng_schedule: already scheduled");
    if (g->nodes.empty()) return g->fail(NG_EINVAL, "ng_schedule: empty graph");
    std::vector<std::pair<int, int>> edges;
    for (int v = 0; v < (int)g->nodes.size(); ++v)
        for (int u : g->nodes[v].preds) edges.emplace_back(u, v);
    compute_schedule((int)g->nodes.size(), edges, g->sched, g->assignment == NG_ASSIGN_EXACT);
    g->trainable = false;
    for (const Node& nd : g->nodes) g->trainable = g->trainable || nd.op == NG_OP_SGD_UPDATE;
    g->phase = SCHEDULED;
    return NG_OK;
}

int ng_schedule_sizes(const ng_graph* g, int* n_nodes, int* n_streams, int* n_chains, int* n_meg_edges,
                      int* n_matching, int* n_sync, int* n_events) {
    if (!g) return NG_EINVAL;
    if (g->phase < SCHEDULED) return const_cast<ng_graph*>(g)->fail(NG_ESTATE, "ng_schedule_sizes: call ng_schedule first");
    const Schedule& s = g->sched;
    if (n_nodes) *n_nodes = (int)g->nodes.size();
    if (n_streams) *n_streams = s.n_streams;
    if (n_chains) *n_chains = s.n_chains;
    if (n_meg_edges) *n_meg_edges = (int)s.meg.size();
    if (n_matching) *n_matching = s.n_matching;
    if (n_sync) *n_sync = (int)s.sync.size();
    if (n_events) *n_events = s.n_events;
    return NG_OK;
}

int ng_get_schedule(const ng_graph* g, int* order, int* stream_of, int* chain_of, int* event_of,
                    int* meg_src, int* meg_dst, int* sync_src, int* sync_dst) {
    if (!g) return NG_EINVAL;
    if (g->phase < SCHEDULED) return const_cast<ng_graph*>(g)->fail(NG_ESTATE, "ng_get_schedule: call ng_schedule first");
    const Schedule& s = g->sched;
    const size_t n = g->nodes.size();
    if (order) std::copy(s.order.begin(), s.order.end(), order);
    if (stream_of) std::copy(s.stream_of.begin(), s.stream_of.end(), stream_of);
    if (chain_of) std::copy(s.chain_of.begin(), s.chain_of.end(), chain_of);
    if (event_of) std::copy(s.event_of.begin(), s.event_of.end(), event_of);
    (void)n;
    for (size_t i = 0; i < s.meg.size(); ++i) {
        if (meg_src) meg_src[i] = s.meg[i].first;
        if (meg_dst) meg_dst[i] = s.meg[i].second;
    }
    for (size_t i = 0; i < s.sync.size(); ++i) {
        if (sync_src) sync_src[i] = s.sync[i].first;
        if (sync_dst) sync_dst[i] = s.sync[i].second;
    }
    return NG_OK;
}

int ng_get_scaffold(const ng_graph* g, int* fork, int* n_fork, int* join, int* n_join) {
    if (!g) return NG_EINVAL;
    if (g->phase < SCHEDULED) return const_cast<ng_graph*>(g)->fail(NG_ESTATE, "ng_get_scaffold: call ng_schedule first");
    const Schedule& s = g->sched;
    if (fork) std::copy(s.fork.begin(), s.fork.end(), fork);
    if (join) std::copy(s.join.begin(), s.join.end(), join);
    if (n_fork) *n_fork = (int)s.fork.size();
    if (n_join) *n_join = (int)s.join.size();
    return NG_OK;
}

int ng_plan_memory(ng_graph* g, size_t* arena_bytes) {
    if (!g) return NG_EINVAL;
    if (g->phase < SCHEDULED) return g->fail(NG_ESTATE, "ng_plan_memory: call ng_schedule first");
    if (g->phase > PLANNED) return g->fail(NG_ESTATE, "ng_plan_memory: already bound");
    const size_t n = g->nodes.size();
    g->offset.assign(n, 0);
    g->bytes.assign(n, 0);
    // A tensor that one concat takes whole (batch 1: a channel block of the result is one
    // contiguous range) is produced in place, inside the concat's buffer; the concat then has
    // nothing to copy for it. Everything else gets a private buffer; nothing is reused.
    g->alias_of.assign(n, -1);
    std::vector<size_t> inside(n, 0);                       // byte offset inside the concat's buffer
    if (!knob("NG_NO_CONCAT_ALIAS"))
        for (size_t c = 0; c < n; ++c) {
            const Node& cat = g->nodes[c];
            if (cat.op != NG_OP_CONCAT || cat.out.n != 1) continue;
            const size_t plane = (size_t)cat.out.h * cat.out.w * sizeof(float);
            size_t first = 0;
            for (size_t j = 0; j < cat.preds.size(); ++j) {
                const int p = cat.preds[j];
                const Node& src = g->nodes[p];
                const bool whole = cat.p.slice_lo[j] == 0 && cat.p.slice_hi[j] == src.out.c;
                const bool once = std::count(cat.preds.begin(), cat.preds.end(), p) == 1;
                if (src.op != NG_OP_INPUT && g->alias_of[p] < 0 && whole && once && (first * plane) % 16 == 0) {
                    g->alias_of[p] = (int)c;
                    inside[p] = first * plane;
                }
                first += (size_t)(cat.p.slice_hi[j] - cat.p.slice_lo[j]);
            }
        }
    size_t top = 0;
    // Reuse over time (optional): a buffer whose tensor is dead can hold a later tensor. With several
    // streams "dead" cannot mean "earlier in the submission order": tensor z is dead for node v only if
    // z's producer and every reader of z are ancestors of v, because only then does every execution
    // that respects the DAG - whatever runs beside whatever - finish them before v starts to write.
    // Network inputs and outputs and the tensors of in-place concats keep private buffers.
    std::vector<std::vector<uint64_t>> anc;     // anc[v]: bit u set iff u is a strict ancestor of v
    std::vector<std::vector<int>> readers(n);
    std::vector<char> shares(n, 0);             // takes part in an in-place concat (as input or as the concat)
    struct Block { size_t offset, bytes; int owner; };
    std::vector<Block> blocks;                  // buffers that may be handed on, with their latest owner
    if (g->memory_reuse) {
        const size_t words = (n + 63) / 64;
        anc.assign(n, std::vector<uint64_t>(words, 0));
        for (size_t v = 0; v < n; ++v)
            for (int u : g->nodes[v].preds) {
                readers[u].push_back((int)v);
                anc[v][u / 64] |= 1ull << (u % 64);
                for (size_t w = 0; w < words; ++w) anc[v][w] |= anc[u][w];
            }
        for (size_t v = 0; v < n; ++v)
            if (g->alias_of[v] >= 0) shares[v] = shares[g->alias_of[v]] = 1;
    }
    auto dead_for = [&](int z, size_t v) {
        if (!((anc[v][z / 64] >> (z % 64)) & 1)) return false;
        for (int r : readers[z])
            if (!((anc[v][r / 64] >> (r % 64)) & 1)) return false;
        return true;
    };
    for (size_t v = 0; v < n; ++v) {            // one buffer per remaining node output, 256-byte aligned
        g->bytes[v] = (size_t)g->nodes[v].out.elems() * sizeof(float);
        if (g->alias_of[v] >= 0) continue;
        const size_t need = (g->bytes[v] + 255) & ~(size_t)255;
        const bool own = !g->memory_reuse || g->nodes[v].op == NG_OP_INPUT || g->nodes[v].is_output || shares[v];
        int pick = -1;
        if (!own)                               // the smallest handed-on buffer that is large enough and dead for v
            for (size_t b = 0; b < blocks.size(); ++b)
                if (blocks[b].bytes >= need && (pick < 0 || blocks[b].bytes < blocks[pick].bytes) && dead_for(blocks[b].owner, v)) pick = (int)b;
        if (pick >= 0) {
            g->offset[v] = blocks[pick].offset;
            blocks[pick].owner = (int)v;
            continue;
        }
        g->offset[v] = top;
        top += need;
        if (!own) blocks.push_back(Block{g->offset[v], need, (int)v});
    }
    for (size_t v = n; v-- > 0;)                // a concat has a higher id than its inputs: its own place is final by now
        if (g->alias_of[v] >= 0) g->offset[v] = g->offset[g->alias_of[v]] + inside[v];
    g->arena_bytes = top;
    g->phase = PLANNED;
    if (arena_bytes) *arena_bytes = top;
    return NG_OK;
}

int ng_set_memory_reuse(ng_graph* g, int on) {
    if (!g) return NG_EINVAL;
    if (g->phase > SCHEDULED) return g->fail(NG_ESTATE, "ng_set_memory_reuse: the memory plan is already made");
    g->memory_reuse = on != 0;
    return NG_OK;
}

int ng_set_launch_fusion(ng_graph* g, int on) {
    if (!g) return NG_EINVAL;
    if (g->phase >= BOUND) return g->fail(NG_ESTATE, "ng_set_launch_fusion: the task table is already built");
    g->launch_fusion = on != 0;
    return NG_OK;
}

int ng_get_offsets(const ng_graph* g, size_t* offset, size_t* bytes) {
    if (!g) return NG_EINVAL;
    if (g->phase < PLANNED) return const_cast<ng_graph*>(g)->fail(NG_ESTATE, "ng_get_offsets: call ng_plan_memory first");
    if (offset) std::copy(g->offset.begin(), g->offset.end(), offset);
    if (bytes) std::copy(g->bytes.begin(), g->bytes.end(), bytes);
    return NG_OK;
}

int ng_critical_path(const ng_graph* g, const float* t, float* total, int* path, int* n_path) {
    if (!g || !t) return NG_EINVAL;
    const int n = (int)g->nodes.size();
    if (n == 0) return NG_EINVAL;
    std::vector<double> best(n);
    std::vector<int> from(n, -1);
    int last = 0;
    for (int v = 0; v < n; ++v) {               // ids are a topological order
        double b = 0;
        for (int u : g->nodes[v].preds)
            if (from[v] < 0 || best[u] > b) {
                b = best[u];
                from[v] = u;
            }
        best[v] = b + t[v];
        if (best[v] > best[last]) last = v;
    }
    std::vector<int> rev;
    for (int v = last; v >= 0; v = from[v]) rev.push_back(v);
    if (total) *total = (float)best[last];
    if (n_path) *n_path = (int)rev.size();
    if (path) std::reverse_copy(rev.begin(), rev.end(), path);
    return NG_OK;
}

int ng_task_work(const ng_graph* g, int id, double* bytes, double* flops) {
    if (!g || id < 0 || id >= (int)g->nodes.size()) return NG_EINVAL;
    const Node& nd = g->nodes[id];
    const double out = (double)nd.out.elems();
    double in0 = nd.preds.empty() ? 0 : (double)g->nodes[nd.preds[0]].out.elems();
    double cin = nd.preds.empty() ? 0 : (double)g->nodes[nd.preds[0]].out.c;
    double b = 0, f = 0;
    switch (nd.op) {
        case NG_OP_CONV1X1: b = 4 * (in0 + cin * nd.out.c + out); f = 2 * cin * out; break;
        case NG_OP_DWCONV: b = 4 * (in0 + nd.out.c * nd.p.k * nd.p.k + out); f = 2.0 * nd.p.k * nd.p.k * out; break;
        case NG_OP_CONV3X3: b = 4 * (in0 + 9 * cin * nd.out.c + out); f = 18 * cin * out; break;
        case NG_OP_BN_ACT: b = 8 * out + 16.0 * nd.out.c; f = 2 * out; break;
        case NG_OP_RELU: b = 8 * out; f = out; break;
        case NG_OP_ADD_N: b = 4 * (nd.preds.size() + 1.0) * out; f = (nd.preds.size() - 1.0) * out; break;
        case NG_OP_CONCAT: b = 8 * out; break;
        case NG_OP_POOL: b = 4 * (in0 + out); f = 9 * out; break;
        case NG_OP_GLOBAL_AVGPOOL: b = 4 * (in0 + out); f = in0; break;
        case NG_OP_FC: b = 4 * (cin * nd.out.c + nd.out.c + in0 + out); f = 2 * cin * out; break;
        // backward operators: in0 = elements of dy, in1 = elements of x
        case NG_OP_CONV1X1_DGRAD: b = 4 * (in0 + cin * nd.out.c + out); f = 2 * cin * out; break;
        case NG_OP_CONV3X3_DGRAD: b = 4 * (in0 + 9 * cin * nd.out.c + out); f = 18.0 * nd.out.c * in0; break;
        case NG_OP_CONV1X1_WGRAD:
        case NG_OP_CONV3X3_WGRAD: {
            const double in1 = (double)g->nodes[nd.preds[1]].out.elems(), cx = (double)g->nodes[nd.preds[1]].out.c;
            b = 4 * (in0 + in1 + out);
            f = 2.0 * cx * in0 * (nd.op == NG_OP_CONV3X3_WGRAD ? 9 : 1);
            break;
        }
        case NG_OP_DWCONV_DGRAD: b = 4 * (in0 + nd.out.c * nd.p.k * nd.p.k + out); f = 2.0 * nd.p.k * nd.p.k * in0; break;
        case NG_OP_DWCONV_WGRAD: b = 4 * (in0 + (double)g->nodes[nd.preds[1]].out.elems() + out); f = 2.0 * nd.p.k * nd.p.k * in0; break;
        case NG_OP_BN_ACT_DGRAD: b = 12 * out + 16.0 * nd.out.c; f = 4 * out; break;
        case NG_OP_BN_ACT_WGRAD: b = 8 * in0 + 16.0 * cin; f = 6 * in0; break;
        case NG_OP_RELU_DGRAD: b = 12 * out; f = out; break;
        case NG_OP_POOL_DGRAD: b = 4 * (in0 + 2 * out); f = 9 * out; break;
        case NG_OP_GAP_DGRAD: b = 4 * (in0 + out); f = out; break;
        case NG_OP_CHANNEL_SUM: b = 4 * (in0 + out); f = in0; break;
        case NG_OP_SLICE_PAD: b = 4 * (out + out); break;
        case NG_OP_SGD_UPDATE: b = 12.0 * nd.p.cout; f = 2.0 * nd.p.cout; break;
        default: break;
    }
    if (bytes) *bytes = b;
    if (flops) *flops = f;
    return NG_OK;
}

}  // extern "C"
