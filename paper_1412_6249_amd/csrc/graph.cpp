// Minimal single-GPU bi-graph executor.
//
// Paper section 2: a network is a directed bipartite graph of tensor and operator vertices; edges
// only join a tensor and an operator. Section 2.1: an operator fires when all its incoming tensors
// are ready, a tensor is ready when all its incoming operators have completed, the computation
// starts at the sources and stops when all sinks are reached. Section 3: operators carry a
// `thread` id - same id, same queue; different ids run in parallel where possible.
//
// On one GPU a `thread` is a HIP stream. Device work is asynchronous, so "completed" for the host
// side bookkeeping means "issued on its stream": readiness is carried onto the device by stream
// order inside a thread and by an event recorded after an operator that a consumer on another
// stream (or a host operator) has to wait for. purine_graph_run returns only after the device work
// behind every sink has finished, which is the synchronisation point that lets graphs be iterated
// (section 2.2); purine_graph_iterate keeps that point on the device between its iterations.
#include <deque>
#include <map>
#include <mutex>
#include <string>
#include <vector>

#include "common.h"

using namespace purine;

struct purine_graph {
    struct Tensor {
        purine_tensor desc;
        std::string name;
        std::vector<int> writers;   // incoming operators
        std::vector<int> readers;   // outgoing operators
    };
    struct Op {
        int kind;
        purine_op_attrs attrs;
        std::vector<int> in, out;
        int thread;
        hipEvent_t done = nullptr;  // recorded after the operator on its stream (device ops only)
        hipEvent_t t0 = nullptr, t1 = nullptr;   // timing bracket around the main kernel
        bool timed = false;
    };
    std::vector<Tensor> tensors;
    std::vector<Op> ops;
    std::map<int, hipStream_t> streams;        // thread id -> stream
    std::map<int, bool> stream_owned;
    std::vector<int> fire_log;
    bool validated = false;
    bool uses_device = false;
    bool timing = false;
    int timing_only = -1;   // >= 0: bracket this operator only, and give it the device to itself
    bool serial = false;    // every operator gets the device to itself
    std::map<int, hipEvent_t> drain;   // per stream: marks the work issued before the exclusive operator
    // Filled by validation from the dispatcher's firing order (which depends on the graph alone):
    // the producers whose completion event operator o has to wait for, and whether anybody waits
    // for operator o's event at all (an event nobody waits for is not recorded).
    std::vector<std::vector<int>> waits;
    std::vector<char> record;
    std::vector<int> plan;   // the firing order itself
    // Replay mode: one pass of the dispatcher recorded into a HIP graph per binding of tensor
    // vertices to storage (the swap step alternates between two of them).
    struct Captured { std::vector<void*> key; hipGraph_t graph; hipGraphExec_t exec; };
    bool replay = false;
    std::vector<Captured> captured;
    hipEvent_t fork = nullptr;
};

namespace {

size_t elem_size(const purine_tensor& t) { return t.dtype == PURINE_BF16 ? 2 : 4; }
size_t image_bytes(const purine_tensor& t) {
    size_t n = 1;
    for (int i = 1; i < t.ndim; ++i) n *= (size_t)t.dim[i];
    return n * elem_size(t);
}
// bytes between consecutive images: more than one image only for a channel-slice view
size_t stride_bytes(const purine_tensor& t) {
    return (t.ndim == 4 && t.nstride != 0) ? (size_t)t.nstride * elem_size(t) : image_bytes(t);
}
// bytes from the first to one past the last element
size_t tensor_bytes(const purine_tensor& t) {
    return ((size_t)t.dim[0] - 1) * stride_bytes(t) + image_bytes(t);
}

// Storage touched by one operand: [lo, hi), and for a channel-slice view the bytes per image and
// the distance between images (0 for anything dense).
struct Range { uintptr_t lo, hi; size_t image = 0, stride = 0; };
Range range_of(const purine_tensor& t) {
    Range r{(uintptr_t)t.data, (uintptr_t)t.data + tensor_bytes(t)};
    if (stride_bytes(t) != image_bytes(t)) { r.image = image_bytes(t); r.stride = stride_bytes(t); }
    return r;
}
// Do the two share a byte? Exact for dense ranges; two views with the same distance between images
// (channel slices of one buffer) are compared per image, modulo that distance; otherwise the spans
// decide (conservative).
bool hit(const Range& a, const Range& b) {
    if (!(a.lo < b.hi && b.lo < a.hi)) return false;
    if (a.stride != 0 && a.stride == b.stride) {
        const size_t s = a.stride;
        const size_t d = a.lo >= b.lo ? (a.lo - b.lo) % s : (s - (b.lo - a.lo) % s) % s;   // (a.lo - b.lo) mod s
        return d < b.image || s - d < a.image;
    }
    return true;
}

bool arity_ok(int kind, int n_in, int n_out, float beta) {
    const int extra = beta != 0.0f ? 1 : 0;
    switch (kind) {
        case PURINE_OP_CONV_FWD: return n_in == 2 && n_out == 1;
        case PURINE_OP_BIAS_FWD: return n_in == 2 && n_out == 1;
        case PURINE_OP_CONV_BWD_DATA: return n_in == 2 + extra && n_out == 1;
        case PURINE_OP_CONV_BWD_WEIGHT: return n_in == 2 + extra && n_out == 1;
        case PURINE_OP_BIAS_BWD: return n_in == 1 + extra && n_out == 1;
        case PURINE_OP_RELU_FWD: return n_in == 1 && n_out == 1;
        case PURINE_OP_RELU_BWD: return n_in == 2 && n_out == 1;
        case PURINE_OP_MAXPOOL_FWD: return n_in == 1 && n_out == 2;
        case PURINE_OP_MAXPOOL_BWD: return n_in == 2 + extra && n_out == 1;
        case PURINE_OP_MAXPOOL_BWD_RELU: return n_in == 3 + extra && n_out == 1;
        case PURINE_OP_CONCAT_FWD: return n_in >= 1 && n_in <= 64 && n_out == 1;
        case PURINE_OP_CONCAT_BWD: return n_in == 1 && n_out >= 1 && n_out <= 64;
        case PURINE_OP_SUM: return n_in >= 1 && n_in <= 8 && n_out == 1;
        case PURINE_OP_HOST_NOP: return n_in >= 0 && n_out >= 0;
        case PURINE_OP_CONV_FWD_BIAS_RELU: return n_in == 3 && n_out == 1;
        case PURINE_OP_CONV_BWD_DATA_RELU: return n_in == 3 + extra && n_out == 1;
        case PURINE_OP_CONV_BWD_WEIGHT_BIAS: return n_in == 2 + 2 * extra && n_out == 2;
        case PURINE_OP_SGD_UPDATE: return n_in == 2 && n_out == 1;
        case PURINE_OP_ALIAS: return n_in >= 1 && n_in <= 64 && n_out >= 1 && n_out <= 64;
        case PURINE_OP_FC_FWD: return n_in == 3 && n_out == 1;
        case PURINE_OP_FC_BWD_DATA: return n_in == 2 && n_out == 1;
        case PURINE_OP_FC_BWD_WEIGHT: return n_in == 2 + 2 * extra && n_out == 2;
        case PURINE_OP_GROUPED_CONV_FWD: return n_in == 3 && n_out == 1;
        case PURINE_OP_GROUPED_CONV_BWD_DATA: return n_in == 2 + extra && n_out == 1;
        case PURINE_OP_GROUPED_CONV_BWD_WEIGHT: return n_in == 2 + 2 * extra && n_out == 2;
        default: return false;
    }
}

// Streams the executor creates itself come from a pool per device that lives as long as the
// process: a graph's k-th thread gets the pool's k-th stream. The runtime spreads streams over a
// few hardware queues in the order they are created, so a process that builds and destroys graphs
// one after another (each with streams of its own) ends up with a graph whose streams share a
// queue and run one behind the other: the same workload measured 5 % slower as the fourth graph of
// a process than as the first. Graphs alive at the same time share these streams, which only adds
// ordering between them.
hipStream_t pooled_stream(int index, int* rc) {
    static std::mutex mu;
    static std::map<int, std::vector<hipStream_t>> pool;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) { *rc = PURINE_E_HIP; return nullptr; }
    std::lock_guard<std::mutex> lock(mu);
    std::vector<hipStream_t>& v = pool[dev];
    while ((int)v.size() <= index) {
        hipStream_t s = nullptr;
        if (hipStreamCreateWithFlags(&s, hipStreamNonBlocking) != hipSuccess) { *rc = PURINE_E_HIP; return nullptr; }
        v.push_back(s);
    }
    return v[index];
}

hipStream_t stream_of(purine_graph* g, int thread, int* rc) {
    auto it = g->streams.find(thread);
    if (it != g->streams.end()) return it->second;
    int owned = 0;
    for (const auto& kv : g->stream_owned) owned += kv.second ? 1 : 0;
    hipStream_t s = pooled_stream(owned, rc);
    if (!s) return nullptr;
    g->streams[thread] = s;
    g->stream_owned[thread] = true;
    return s;
}

void drop_captured(purine_graph* g) {
    for (auto& c : g->captured) {
        if (c.exec) (void)hipGraphExecDestroy(c.exec);
        if (c.graph) (void)hipGraphDestroy(c.graph);
    }
    g->captured.clear();
}

// The dispatcher of section 2.1 as host bookkeeping: an operator is queued on its thread when all
// its incoming tensors are ready, a tensor is ready when all its incoming operators have fired, one
// operator per thread queue fires per sweep so that independent threads interleave. fire(o) returns
// a status; the walk stops at the first error. Returns how many operators fired.
template <class Fire>
int dispatch(const purine_graph* g, Fire&& fire, int* rc) {
    const int no = (int)g->ops.size(), nt = (int)g->tensors.size();
    std::vector<int> inputs_pending(no), writers_pending(nt);
    for (int t = 0; t < nt; ++t) writers_pending[t] = (int)g->tensors[t].writers.size();
    std::map<int, std::deque<int>> queues;      // thread id -> FIFO of operators ready to fire
    for (int o = 0; o < no; ++o) {
        int pend = 0;
        for (int t : g->ops[o].in) if (writers_pending[t] > 0) ++pend;
        inputs_pending[o] = pend;
    }
    for (int o = 0; o < no; ++o)
        if (inputs_pending[o] == 0) queues[g->ops[o].thread].push_back(o);   // fed by source tensors only
    int fired = 0;
    bool progress = true;
    *rc = PURINE_OK;
    while (fired < no && progress) {
        progress = false;
        for (auto& kv : queues) {
            if (kv.second.empty()) continue;
            const int o = kv.second.front();
            kv.second.pop_front();
            if ((*rc = fire(o)) != PURINE_OK) return fired;
            ++fired;
            progress = true;
            // the operator has completed as far as the dispatcher is concerned: update its outgoing tensors
            for (int t : g->ops[o].out)
                if (--writers_pending[t] == 0)
                    for (int rd : g->tensors[t].readers)
                        if (--inputs_pending[rd] == 0) queues[g->ops[rd].thread].push_back(rd);
        }
    }
    return fired;
}

// Issues one device operator on `st`. Storage identity rules of the in-place forms are checked here.
int issue(purine_graph* g, purine_graph::Op& op, hipStream_t st) {
    auto T = [&](int id) -> purine_tensor* { return &g->tensors[id].desc; };
    const purine_op_attrs& a = op.attrs;
    switch (op.kind) {
        case PURINE_OP_CONV_FWD:
            return purine_conv_fwd(&a.conv, T(op.in[0]), T(op.in[1]), T(op.out[0]), a.ws, a.ws_bytes, st);
        case PURINE_OP_CONV_FWD_BIAS_RELU:
            return purine_conv_fwd_bias_relu(&a.conv, T(op.in[0]), T(op.in[1]), T(op.in[2]), T(op.out[0]),
                                             a.relu, a.ws, a.ws_bytes, st);
        case PURINE_OP_CONV_BWD_DATA_RELU:
            if (a.beta != 0.0f && T(op.in[3])->data != T(op.out[0])->data) return PURINE_E_LAYOUT;
            return purine_conv_bwd_data_relu(&a.conv, T(op.in[0]), T(op.in[1]), T(op.in[2]), T(op.out[0]),
                                             a.beta, a.ws, a.ws_bytes, st);
        case PURINE_OP_BIAS_FWD:
            if (T(op.in[0])->data != T(op.out[0])->data) return PURINE_E_LAYOUT;
            return purine_bias_fwd(T(op.in[1]), T(op.out[0]), st);
        case PURINE_OP_CONV_BWD_DATA:
            if (a.beta != 0.0f && T(op.in[2])->data != T(op.out[0])->data) return PURINE_E_LAYOUT;
            return purine_conv_bwd_data(&a.conv, T(op.in[0]), T(op.in[1]), T(op.out[0]), a.beta, a.ws, a.ws_bytes, st);
        case PURINE_OP_CONV_BWD_WEIGHT:
            if (a.beta != 0.0f && T(op.in[2])->data != T(op.out[0])->data) return PURINE_E_LAYOUT;
            return purine_conv_bwd_weight(&a.conv, T(op.in[0]), T(op.in[1]), T(op.out[0]), a.beta, a.ws, a.ws_bytes, st);
        case PURINE_OP_CONV_BWD_WEIGHT_BIAS:
            if (a.beta != 0.0f && (T(op.in[2])->data != T(op.out[0])->data || T(op.in[3])->data != T(op.out[1])->data))
                return PURINE_E_LAYOUT;
            return purine_conv_bwd_weight_bias(&a.conv, T(op.in[0]), T(op.in[1]), T(op.out[0]), T(op.out[1]),
                                               a.beta, a.ws, a.ws_bytes, st);
        case PURINE_OP_BIAS_BWD:
            if (a.beta != 0.0f && T(op.in[1])->data != T(op.out[0])->data) return PURINE_E_LAYOUT;
            return purine_bias_bwd(T(op.in[0]), T(op.out[0]), a.beta, a.ws, a.ws_bytes, st);
        case PURINE_OP_ALIAS:
            return PURINE_OK;   // names existing storage; ordering is all it contributes
        case PURINE_OP_FC_FWD:
            return purine_fc_fwd(T(op.in[0]), T(op.in[1]), T(op.in[2]), T(op.out[0]), a.ws, a.ws_bytes, st);
        case PURINE_OP_FC_BWD_DATA:
            return purine_fc_bwd_data(T(op.in[0]), T(op.in[1]), T(op.out[0]), a.ws, a.ws_bytes, st);
        case PURINE_OP_FC_BWD_WEIGHT:
            if (a.beta != 0.0f && (T(op.in[2])->data != T(op.out[0])->data || T(op.in[3])->data != T(op.out[1])->data))
                return PURINE_E_LAYOUT;
            return purine_fc_bwd_weight(T(op.in[0]), T(op.in[1]), T(op.out[0]), T(op.out[1]), a.beta, a.ws, a.ws_bytes, st);
        case PURINE_OP_GROUPED_CONV_FWD:
            return purine_grouped_conv_fwd(&a.conv, a.groups ? a.groups : 1, T(op.in[0]), T(op.in[1]), T(op.in[2]),
                                           T(op.out[0]), a.relu, a.ws, a.ws_bytes, st);
        case PURINE_OP_GROUPED_CONV_BWD_DATA:
            if (a.beta != 0.0f && T(op.in[2])->data != T(op.out[0])->data) return PURINE_E_LAYOUT;
            return purine_grouped_conv_bwd_data(&a.conv, a.groups ? a.groups : 1, T(op.in[0]), T(op.in[1]), T(op.out[0]),
                                                a.beta, a.ws, a.ws_bytes, st);
        case PURINE_OP_GROUPED_CONV_BWD_WEIGHT:
            if (a.beta != 0.0f && (T(op.in[2])->data != T(op.out[0])->data || T(op.in[3])->data != T(op.out[1])->data))
                return PURINE_E_LAYOUT;
            return purine_grouped_conv_bwd_weight(&a.conv, a.groups ? a.groups : 1, T(op.in[0]), T(op.in[1]), T(op.out[0]),
                                                  T(op.out[1]), a.beta, a.ws, a.ws_bytes, st);
        case PURINE_OP_SGD_UPDATE:
            return purine_sgd_update(T(op.in[0]), T(op.in[1]), T(op.out[0]), a.lr, st);
        case PURINE_OP_RELU_FWD:
            return purine_relu_fwd(T(op.in[0]), T(op.out[0]), st);
        case PURINE_OP_RELU_BWD:
            return purine_relu_bwd(T(op.in[0]), T(op.in[1]), T(op.out[0]), st);
        case PURINE_OP_MAXPOOL_FWD:
            return purine_maxpool_fwd(&a.pool, T(op.in[0]), T(op.out[0]), T(op.out[1]), st);
        case PURINE_OP_MAXPOOL_BWD:
            if (a.beta != 0.0f && T(op.in[2])->data != T(op.out[0])->data) return PURINE_E_LAYOUT;
            return purine_maxpool_bwd(&a.pool, T(op.in[0]), T(op.in[1]), T(op.out[0]), a.beta, st);
        case PURINE_OP_MAXPOOL_BWD_RELU:
            if (a.beta != 0.0f && T(op.in[3])->data != T(op.out[0])->data) return PURINE_E_LAYOUT;
            return purine_maxpool_bwd_relu(&a.pool, T(op.in[0]), T(op.in[1]), T(op.in[2]), T(op.out[0]), a.beta, st);
        case PURINE_OP_CONCAT_FWD: {
            std::vector<const purine_tensor*> parts;
            for (int id : op.in) parts.push_back(T(id));
            return purine_concat_fwd(parts.data(), (int)parts.size(), T(op.out[0]), st);
        }
        case PURINE_OP_CONCAT_BWD: {
            std::vector<purine_tensor*> parts;
            for (int id : op.out) parts.push_back(T(id));
            return purine_concat_bwd(T(op.in[0]), parts.data(), (int)parts.size(), st);
        }
        case PURINE_OP_SUM: {
            std::vector<const purine_tensor*> terms;
            for (int id : op.in) terms.push_back(T(id));
            return purine_sum(terms.data(), (int)terms.size(), T(op.out[0]), st);
        }
        default:
            return PURINE_E_ARG;
    }
}

}  // namespace

extern "C" {

purine_graph* purine_graph_create(void) { return new (std::nothrow) purine_graph(); }

void purine_graph_destroy(purine_graph* g) {
    if (!g) return;
    for (auto& op : g->ops)
    {
        if (op.done) (void)hipEventDestroy(op.done);
        if (op.t0) (void)hipEventDestroy(op.t0);
        if (op.t1) (void)hipEventDestroy(op.t1);
    }
    drop_captured(g);
    if (g->fork) (void)hipEventDestroy(g->fork);
    for (auto& kv : g->drain) if (kv.second) (void)hipEventDestroy(kv.second);
    delete g;                                  // (its own streams belong to the pool)
}

int purine_graph_add_tensor(purine_graph* g, const purine_tensor* t, const char* name) {
    if (!g || !t) return PURINE_E_NULL;
    if (t->ndim < 1 || t->ndim > 4) return PURINE_E_SHAPE;
    for (int i = 0; i < t->ndim; ++i)
        if (t->dim[i] < 1) return PURINE_E_SHAPE;
    if (t->dtype != PURINE_F32 && t->dtype != PURINE_BF16 && t->dtype != PURINE_I32) return PURINE_E_DTYPE;
    if (t->nstride != 0 && (t->ndim != 4 || t->nstride < t->dim[1] * t->dim[2] * t->dim[3])) return PURINE_E_SHAPE;
    purine_graph::Tensor v;
    v.desc = *t;
    if (name) v.name = name;
    g->tensors.push_back(v);
    g->validated = false;
    drop_captured(g);
    return (int)g->tensors.size() - 1;
}

int purine_graph_add_op(purine_graph* g, int op_kind, const purine_op_attrs* attrs,
                        const int* in_ids, int n_in, const int* out_ids, int n_out, int thread_id) {
    if (!g) return PURINE_E_NULL;
    if (n_in < 0 || n_out < 0 || thread_id < 0) return PURINE_E_ARG;
    if ((n_in > 0 && !in_ids) || (n_out > 0 && !out_ids)) return PURINE_E_NULL;
    purine_graph::Op op;
    op.kind = op_kind;
    op.attrs = purine_op_attrs{};
    if (attrs) op.attrs = *attrs;
    if (!arity_ok(op_kind, n_in, n_out, op.attrs.beta)) return PURINE_E_ARG;
    const int nt = (int)g->tensors.size();
    for (int i = 0; i < n_in; ++i) {
        if (in_ids[i] < 0 || in_ids[i] >= nt) return PURINE_E_ARG;
        op.in.push_back(in_ids[i]);
    }
    for (int i = 0; i < n_out; ++i) {
        if (out_ids[i] < 0 || out_ids[i] >= nt) return PURINE_E_ARG;
        for (int j = 0; j < n_in; ++j)
            if (in_ids[j] == out_ids[i]) return PURINE_E_GRAPH;   // a self loop through one vertex
        for (int j = 0; j < i; ++j)
            if (out_ids[j] == out_ids[i]) return PURINE_E_GRAPH;
        op.out.push_back(out_ids[i]);
    }
    if (op_kind == PURINE_OP_ALIAS) {
        // every output lies inside the span of the inputs
        uintptr_t lo = UINTPTR_MAX, hi = 0;
        for (int t : op.in) {
            const purine_tensor& d = g->tensors[t].desc;
            if (!d.data) return PURINE_E_NULL;
            const Range r = range_of(d);
            lo = r.lo < lo ? r.lo : lo;
            hi = r.hi > hi ? r.hi : hi;
        }
        for (int t : op.out) {
            const purine_tensor& d = g->tensors[t].desc;
            if (!d.data) return PURINE_E_NULL;
            const Range r = range_of(d);
            if (r.lo < lo || r.hi > hi) return PURINE_E_LAYOUT;
        }
    }
    op.thread = thread_id;
    const int id = (int)g->ops.size();
    g->ops.push_back(op);
    for (int t : g->ops[id].in) g->tensors[t].readers.push_back(id);
    for (int t : g->ops[id].out) g->tensors[t].writers.push_back(id);
    if (op_kind != PURINE_OP_HOST_NOP) g->uses_device = true;
    g->validated = false;
    drop_captured(g);
    return id;
}

int purine_graph_set_stream(purine_graph* g, int thread_id, void* hip_stream) {
    if (!g) return PURINE_E_NULL;
    if (thread_id < 0) return PURINE_E_ARG;
    g->streams[thread_id] = (hipStream_t)hip_stream;
    g->stream_owned[thread_id] = false;
    drop_captured(g);
    return PURINE_OK;
}

int purine_graph_validate(purine_graph* g) {
    if (!g) return PURINE_E_NULL;
    const int no = (int)g->ops.size();
    // operator-level successor lists: a -> b when b reads a tensor that a writes
    std::vector<std::vector<int>> succ(no);
    std::vector<int> indeg(no, 0);
    for (int a = 0; a < no; ++a)
        for (int t : g->ops[a].out)
            for (int b : g->tensors[t].readers) { succ[a].push_back(b); ++indeg[b]; }
    // acyclic?  (Kahn)
    std::vector<int> order;
    {
        std::vector<int> deg = indeg;
        std::deque<int> q;
        for (int a = 0; a < no; ++a) if (deg[a] == 0) q.push_back(a);
        while (!q.empty()) {
            int a = q.front(); q.pop_front();
            order.push_back(a);
            for (int b : succ[a]) if (--deg[b] == 0) q.push_back(b);
        }
        if ((int)order.size() != no) return PURINE_E_GRAPH;
    }
    // reach[a][b]: a path a -> ... -> b exists (bitsets, reverse topological sweep)
    const int words = (no + 63) / 64;
    std::vector<uint64_t> reach((size_t)no * words, 0);
    for (int idx = no - 1; idx >= 0; --idx) {
        const int a = order[idx];
        uint64_t* ra = &reach[(size_t)a * words];
        for (int b : succ[a]) {
            ra[b / 64] |= 1ull << (b % 64);
            const uint64_t* rb = &reach[(size_t)b * words];
            for (int w = 0; w < words; ++w) ra[w] |= rb[w];
        }
    }
    auto ordered = [&](int a, int b) {
        return ((reach[(size_t)a * words + b / 64] >> (b % 64)) & 1) ||
               ((reach[(size_t)b * words + a / 64] >> (a % 64)) & 1);
    };
    // storage hazards: a writer and any other toucher of overlapping bytes must be ordered
    struct Touch { int op; Range r; bool write; };
    std::vector<Touch> touches;
    for (int a = 0; a < no; ++a) {
        const auto& op = g->ops[a];
        if (op.kind == PURINE_OP_HOST_NOP || op.kind == PURINE_OP_ALIAS) continue;   // touch no device storage
        for (int t : op.in) {
            const auto& d = g->tensors[t].desc;
            if (d.data) touches.push_back({a, range_of(d), false});
        }
        for (int t : op.out) {
            const auto& d = g->tensors[t].desc;
            if (d.data) touches.push_back({a, range_of(d), true});
        }
        if (op.attrs.ws && op.attrs.ws_bytes)
            touches.push_back({a, {(uintptr_t)op.attrs.ws, (uintptr_t)op.attrs.ws + op.attrs.ws_bytes}, true});
    }
    for (size_t i = 0; i < touches.size(); ++i)
        for (size_t j = i + 1; j < touches.size(); ++j) {
            const Touch &x = touches[i], &y = touches[j];
            if (x.op == y.op || !(x.write || y.write) || !hit(x.r, y.r)) continue;
            if (!ordered(x.op, y.op)) return PURINE_E_GRAPH;
        }
    // Which completion events are needed. Streams are FIFO, so of an operator's producers on one
    // other stream only the one issued last has to be waited for, and not even that one when an
    // earlier operator of the consumer's stream has already waited for it or for a later one.
    g->waits.assign(no, {});
    g->record.assign(no, 0);
    g->plan.clear();
    {
        std::vector<int> issued(no, -1);
        std::map<std::pair<int, int>, int> covered;   // (consumer thread, producer thread) -> issue index waited for
        int n = 0, rc = PURINE_OK;
        const int fired = dispatch(g, [&](int o) {
            const auto& op = g->ops[o];
            issued[o] = n++;
            g->plan.push_back(o);
            std::map<int, int> last;   // producer thread -> its producer issued last
            for (int t : op.in)
                for (int wr : g->tensors[t].writers) {
                    const auto& w = g->ops[wr];
                    if (w.kind == PURINE_OP_HOST_NOP) continue;          // completes on the host before this fires
                    if (op.kind == PURINE_OP_HOST_NOP) {                  // the host waits for every device producer
                        g->waits[o].push_back(wr);
                        g->record[wr] = 1;
                        continue;
                    }
                    if (w.thread == op.thread) continue;
                    auto it = last.find(w.thread);
                    if (it == last.end() || issued[it->second] < issued[wr]) last[w.thread] = wr;
                }
            for (const auto& kv : last) {
                const auto key = std::make_pair(op.thread, kv.first);
                auto it = covered.find(key);
                if (it != covered.end() && it->second >= issued[kv.second]) continue;
                covered[key] = issued[kv.second];
                g->waits[o].push_back(kv.second);
                g->record[kv.second] = 1;
            }
            return (int)PURINE_OK;
        }, &rc);
        if (fired < no) return PURINE_E_GRAPH;   // some operator can never fire
    }
    g->validated = true;
    return PURINE_OK;
}

namespace {

// Every stream of the graph waits for everything issued so far on all the others: a barrier between
// two runs that the device keeps, without the host waiting.
int join_streams(purine_graph* g) {
    if (g->streams.size() < 2) return PURINE_OK;
    for (auto& sk : g->streams) {
        hipEvent_t& ev = g->drain[sk.first];
        if ((!ev && hipEventCreateWithFlags(&ev, hipEventDisableTiming) != hipSuccess) ||
            hipEventRecord(ev, sk.second) != hipSuccess) return PURINE_E_HIP;
    }
    for (auto& sk : g->streams)
        for (auto& other : g->streams)
            if (other.first != sk.first && hipStreamWaitEvent(sk.second, g->drain[other.first], 0) != hipSuccess)
                return PURINE_E_HIP;
    return PURINE_OK;
}

int wait_streams(purine_graph* g) {
    int rc = PURINE_OK;
    if (g->uses_device)
        for (auto& kv : g->streams)
            if (hipStreamSynchronize(kv.second) != hipSuccess) rc = PURINE_E_HIP;
    return rc;
}

// One pass of the dispatcher over the graph, issuing device work; the host does not wait for it.
int run_issue(purine_graph* g) {
    if (!g->validated) {
        int rc = purine_graph_validate(g);
        if (rc != PURINE_OK) return rc;
    }
    const int no = (int)g->ops.size();
    g->fire_log.clear();
    int rc = PURINE_OK;
    const int fired = dispatch(g, [&](int o) {
        purine_graph::Op& op = g->ops[o];
        int op_rc = PURINE_OK;
        if (op.kind != PURINE_OP_HOST_NOP) {
            hipStream_t st = stream_of(g, op.thread, &op_rc);
            if (op_rc != PURINE_OK) return op_rc;
            // wait for producers that ran on other streams
            for (int wr : g->waits[o])
                if (hipStreamWaitEvent(st, g->ops[wr].done, 0) != hipSuccess) return (int)PURINE_E_HIP;
            op.timed = false;
            const bool timed_op = g->timing && (g->timing_only < 0 || g->timing_only == o) &&
                                  op.kind != PURINE_OP_ALIAS;   // launches nothing to bracket
            const bool exclusive = g->serial || (g->timing && g->timing_only == o);
            if (exclusive) {
                // the one measured operator runs alone: its stream waits for everything issued so
                // far on the other streams, and (below) they wait for it
                for (auto& sk : g->streams) {
                    if (sk.first == op.thread) continue;
                    hipEvent_t& ev = g->drain[sk.first];
                    if ((!ev && hipEventCreateWithFlags(&ev, hipEventDisableTiming) != hipSuccess) ||
                        hipEventRecord(ev, sk.second) != hipSuccess ||
                        hipStreamWaitEvent(st, ev, 0) != hipSuccess) return (int)PURINE_E_HIP;
                }
            }
            if (timed_op) {
                if ((!op.t0 && hipEventCreate(&op.t0) != hipSuccess) ||
                    (!op.t1 && hipEventCreate(&op.t1) != hipSuccess)) return (int)PURINE_E_HIP;
                purine_set_kernel_probe(op.t0, op.t1);
            }
            op_rc = issue(g, op, st);
            if (timed_op) { purine_set_kernel_probe(nullptr, nullptr); op.timed = op_rc == PURINE_OK; }
            if (op_rc != PURINE_OK) return op_rc;
            if (g->record[o] || exclusive) {
                if (!op.done && hipEventCreateWithFlags(&op.done, hipEventDisableTiming) != hipSuccess) return (int)PURINE_E_HIP;
                if (hipEventRecord(op.done, st) != hipSuccess) return (int)PURINE_E_HIP;
            }
            if (exclusive)
                for (auto& sk : g->streams)
                    if (sk.first != op.thread && hipStreamWaitEvent(sk.second, op.done, 0) != hipSuccess) return (int)PURINE_E_HIP;
        } else {
            // a host operator completes on the host: wait for the device producers it consumes, so
            // that readiness keeps its meaning for whatever depends on this operator
            for (int wr : g->waits[o])
                if (hipEventSynchronize(g->ops[wr].done) != hipSuccess) return (int)PURINE_E_HIP;
        }
        g->fire_log.push_back(o);
        return (int)PURINE_OK;
    }, &rc);
    if (rc != PURINE_OK) return rc;
    return fired < no ? PURINE_E_GRAPH : PURINE_OK;
}

// Replay applies to a pass that is all device work on streams of the graph's own, issued the
// plain way (no brackets, no exclusive operators); anything else is issued directly.
bool replay_applies(const purine_graph* g) {
    if (!g->replay || !g->uses_device || g->timing || g->serial) return false;
    for (const auto& op : g->ops)
        if (op.kind == PURINE_OP_HOST_NOP) return false;
    for (const auto& kv : g->stream_owned)
        if (!kv.second) return false;
    return true;
}

// Records one pass of the dispatcher into a HIP graph: the first stream is the origin of the
// capture, the others join it through an event at the start and hand their tails back through an
// event at the end, so the completion events between operators become edges of the graph.
int capture_pass(purine_graph* g, purine_graph::Captured* out) {
    int rc = PURINE_OK;
    for (const auto& op : g->ops) {           // every stream must exist before the capture starts
        (void)stream_of(g, op.thread, &rc);
        if (rc != PURINE_OK) return rc;
    }
    hipStream_t origin = g->streams.begin()->second;
    if (!g->fork && hipEventCreateWithFlags(&g->fork, hipEventDisableTiming) != hipSuccess) return PURINE_E_HIP;
    for (auto& sk : g->streams) {
        hipEvent_t& ev = g->drain[sk.first];
        if (!ev && hipEventCreateWithFlags(&ev, hipEventDisableTiming) != hipSuccess) return PURINE_E_HIP;
    }
    if (hipStreamBeginCapture(origin, hipStreamCaptureModeRelaxed) != hipSuccess) return PURINE_E_HIP;
    bool ok = hipEventRecord(g->fork, origin) == hipSuccess;
    for (auto& sk : g->streams)
        if (ok && sk.second != origin) ok = hipStreamWaitEvent(sk.second, g->fork, 0) == hipSuccess;
    rc = ok ? run_issue(g) : PURINE_E_HIP;
    for (auto& sk : g->streams) {
        if (sk.second == origin) continue;
        hipEvent_t ev = g->drain[sk.first];
        if (hipEventRecord(ev, sk.second) != hipSuccess || hipStreamWaitEvent(origin, ev, 0) != hipSuccess)
            rc = rc != PURINE_OK ? rc : PURINE_E_HIP;
    }
    hipGraph_t graph = nullptr;
    const hipError_t e = hipStreamEndCapture(origin, &graph);   // ends the capture also after an error
    if (rc == PURINE_OK && (e != hipSuccess || !graph)) rc = PURINE_E_HIP;
    hipGraphExec_t exec = nullptr;
    if (rc == PURINE_OK && hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0) != hipSuccess) rc = PURINE_E_HIP;
    if (rc != PURINE_OK) {
        if (graph) (void)hipGraphDestroy(graph);
        (void)hipGetLastError();
        return rc;
    }
    out->graph = graph;
    out->exec = exec;
    return PURINE_OK;
}

// Launches the recorded pass for the current binding of vertices to storage (recording it first
// if there is none yet) on the origin stream. The host does not wait.
int replay_pass(purine_graph* g) {
    if (!g->validated) {
        int rc = purine_graph_validate(g);
        if (rc != PURINE_OK) return rc;
    }
    std::vector<void*> key;
    key.reserve(g->tensors.size());
    for (const auto& t : g->tensors) key.push_back(t.desc.data);
    purine_graph::Captured* hit = nullptr;
    for (auto& c : g->captured)
        if (c.key == key) hit = &c;
    if (!hit) {
        if (g->captured.size() >= 4) drop_captured(g);   // a swap cycle has two bindings; this is a bound
        purine_graph::Captured c{key, nullptr, nullptr};
        const int rc = capture_pass(g, &c);
        if (rc != PURINE_OK) return rc;
        g->captured.push_back(c);
        hit = &g->captured.back();
    }
    return hipGraphLaunch(hit->exec, g->streams.begin()->second) == hipSuccess ? PURINE_OK : PURINE_E_HIP;
}

}  // namespace

int purine_graph_run(purine_graph* g) {
    if (!g) return PURINE_E_NULL;
    const int rc = replay_applies(g) ? replay_pass(g) : run_issue(g);
    // all sinks reached: wait for the device work behind them (every stream the run used)
    const int sync_rc = wait_streams(g);
    return rc != PURINE_OK ? rc : sync_rc;
}

int purine_graph_set_replay(purine_graph* g, int on) {
    if (!g) return PURINE_E_NULL;
    g->replay = on != 0;
    if (!g->replay) drop_captured(g);
    return PURINE_OK;
}

int purine_graph_swap_storage(purine_graph* g, int tensor_a, int tensor_b) {
    if (!g) return PURINE_E_NULL;
    const int nt = (int)g->tensors.size();
    if (tensor_a < 0 || tensor_a >= nt || tensor_b < 0 || tensor_b >= nt || tensor_a == tensor_b) return PURINE_E_ARG;
    const purine_tensor& A = g->tensors[tensor_a].desc;
    const purine_tensor& B = g->tensors[tensor_b].desc;
    if (A.dtype != B.dtype || A.ndim != B.ndim) return PURINE_E_SHAPE;
    for (int i = 0; i < A.ndim; ++i) if (A.dim[i] != B.dim[i]) return PURINE_E_SHAPE;
    if (!A.data || !B.data) return PURINE_E_NULL;
    void* const pa = A.data;
    void* const pb = B.data;
    if (A.nstride != 0 || B.nstride != 0) return PURINE_E_LAYOUT;   // whole buffers only, not channel slices
    const Range ra{(uintptr_t)pa, (uintptr_t)pa + tensor_bytes(A)}, rb{(uintptr_t)pb, (uintptr_t)pb + tensor_bytes(B)};
    if (hit(ra, rb)) return PURINE_E_LAYOUT;
    // The exchange renames two storage ranges. It leaves the set of conflicting operator pairs as
    // it was (so the graph stays valid) only if everything that touches one of the ranges covers
    // exactly that range.
    auto clean = [&](const Range& r) {
        return (!hit(r, ra) || (r.lo == ra.lo && r.hi == ra.hi)) && (!hit(r, rb) || (r.lo == rb.lo && r.hi == rb.hi));
    };
    for (const auto& t : g->tensors)
        if (t.desc.data && !clean(range_of(t.desc))) return PURINE_E_LAYOUT;
    for (const auto& op : g->ops)
        if (op.attrs.ws && op.attrs.ws_bytes) {
            const Range r{(uintptr_t)op.attrs.ws, (uintptr_t)op.attrs.ws + op.attrs.ws_bytes};
            if (hit(r, ra) || hit(r, rb)) return PURINE_E_LAYOUT;
        }
    for (auto& t : g->tensors) {
        if (t.desc.data == pa) t.desc.data = pb;
        else if (t.desc.data == pb) t.desc.data = pa;
    }
    return PURINE_OK;
}

void* purine_graph_tensor_data(const purine_graph* g, int tensor_id) {
    if (!g || tensor_id < 0 || tensor_id >= (int)g->tensors.size()) return nullptr;
    return g->tensors[tensor_id].desc.data;
}

int purine_graph_iterate(purine_graph* g, int n_iters, const int* swap_a, const int* swap_b, int n_swaps) {
    if (!g) return PURINE_E_NULL;
    if (n_iters < 0 || n_swaps < 0 || (n_swaps > 0 && (!swap_a || !swap_b))) return PURINE_E_ARG;
    // Between two iterations the synchronisation point is kept by the device (every stream waits for
    // all the others), not by the host, which runs ahead issuing the next iteration; the kernels of
    // an iteration were issued with the addresses bound at that moment, so the swap is safe.
    int rc = PURINE_OK;
    const bool replay = replay_applies(g);   // recorded passes follow each other on one stream: no join needed
    for (int it = 0; it < n_iters && rc == PURINE_OK; ++it) {
        if (it > 0 && !replay) rc = join_streams(g);
        if (rc == PURINE_OK) rc = replay ? replay_pass(g) : run_issue(g);
        for (int s = 0; s < n_swaps && rc == PURINE_OK; ++s) rc = purine_graph_swap_storage(g, swap_a[s], swap_b[s]);
    }
    const int sync_rc = wait_streams(g);
    return rc != PURINE_OK ? rc : sync_rc;
}

int purine_graph_enable_timing(purine_graph* g, int on) {
    if (!g) return PURINE_E_NULL;
    g->timing = on != 0;
    g->timing_only = -1;
    return PURINE_OK;
}

int purine_graph_set_serial(purine_graph* g, int on) {
    if (!g) return PURINE_E_NULL;
    g->serial = on != 0;
    return PURINE_OK;
}

int purine_graph_time_only(purine_graph* g, int op_id) {
    if (!g) return PURINE_E_NULL;
    if (op_id < 0 || op_id >= (int)g->ops.size()) return PURINE_E_ARG;
    g->timing = true;
    g->timing_only = op_id;
    return PURINE_OK;
}

int purine_graph_op_elapsed_ms(purine_graph* g, int op_id, float* ms) {
    if (!g || !ms) return PURINE_E_NULL;
    if (op_id < 0 || op_id >= (int)g->ops.size()) return PURINE_E_ARG;
    purine_graph::Op& op = g->ops[op_id];
    if (!op.timed || !op.t0 || !op.t1) return PURINE_E_ARG;
    return hipEventElapsedTime(ms, op.t0, op.t1) == hipSuccess ? PURINE_OK : PURINE_E_HIP;
}

int purine_graph_issue_plan(const purine_graph* g, int* op_ids, int cap) {
    if (!g) return PURINE_E_NULL;
    if (!g->validated) return PURINE_E_GRAPH;
    const int n = (int)g->plan.size();
    if (op_ids)
        for (int i = 0; i < n && i < cap; ++i) op_ids[i] = g->plan[i];
    return n;
}

int purine_graph_op_waits(const purine_graph* g, int op_id, int* producer_ids, int cap) {
    if (!g) return PURINE_E_NULL;
    if (!g->validated) return PURINE_E_GRAPH;
    if (op_id < 0 || op_id >= (int)g->ops.size()) return PURINE_E_ARG;
    const auto& w = g->waits[op_id];
    const int n = (int)w.size();
    if (producer_ids)
        for (int i = 0; i < n && i < cap; ++i) producer_ids[i] = w[i];
    return n;
}

int purine_graph_fire_log(const purine_graph* g, int* op_ids, int cap) {
    if (!g) return PURINE_E_NULL;
    const int n = (int)g->fire_log.size();
    if (op_ids)
        for (int i = 0; i < n && i < cap; ++i) op_ids[i] = g->fire_log[i];
    return n;
}

int purine_graph_num_ops(const purine_graph* g) { return g ? (int)g->ops.size() : PURINE_E_NULL; }
int purine_graph_num_tensors(const purine_graph* g) { return g ? (int)g->tensors.size() : PURINE_E_NULL; }

}  // extern "C"
