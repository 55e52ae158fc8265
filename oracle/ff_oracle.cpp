// CPU oracle for the execution simulator of "Beyond Data and Model Parallelism for Deep
// Neural Networks" (FlexFlow), Section 5.
//
// TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition the GPU library is
// checked against.  Only tests, the smoke check and the bench's cpu_baseline leg may call
// it; it shares no code, header or table with the GPU path.
//
// What it computes
//   build   : the task graph of Section 5.1 -- step 1 (one compute task per part of every
//             op's configuration, Section 4) and step 2 (for every tensor edge, every
//             producer-part / consumer-part pair that shares a sub-tensor: a dependency
//             if both parts sit on the same device, otherwise a communication task on the
//             link device between them, assumption A2 for its time).
//   simulate: the full simulation of Section 5.2 (Algorithm 1): READY tasks leave one global
//             queue in (readyTime, task id) order; a dequeued task starts once its device has
//             finished the task dequeued for it before (assumptions A3, A4).
// Delta simulation (Algorithm 2) is defined by the paper to produce the same timeline as a
// full simulation of the changed strategy (Section 5.3), so the oracle for it is: change the
// strategy, build, simulate.
//
// Readings where the paper is silent (all listed in the design notes of this repo):
//   task id = construction order: compute tasks (op order, part index row-major with dim 0
//   slowest), then communication tasks in (edge, producer part, consumer part) order;
//   times are unsigned 64-bit integer ns; part p of a dim of extent E split deg ways covers
//   [floor(p*E/deg), floor((p+1)*E/deg)); device of part k = (offset + k*stride) mod D;
//   link device rows: D + node*G*G + ls*G + lt inside a node (one per ordered GPU pair),
//   D + N*G*G + a*N + b between nodes a != b (one per ordered node pair);
//   transfer time = ceil(bytes / bandwidth) + latency;
//   tensor edges are listed producer by producer (src_op never decreases along the list), so that
//   "communication tasks in edge order" and "op by op" are the same order; other lists are refused
//   (ffo_graph_ok).
//
// Pins: tests/test_oracle_*.py (closed forms, bounds, brute force over task orders, a
// timeline verifier, hand-computed cases under tests/golden/).

#include <algorithm>
#include <cstdint>
#include <cstring>
#include <set>
#include <thread>
#include <utility>
#include <vector>

namespace {

struct DimMap { int8_t src_dim; uint8_t kind; uint16_t stride; int32_t a, b; };   // kind: 0 the consumer reads, 1 the producer contributes
struct Op { uint8_t ndim; uint8_t par_mask; uint16_t type; uint32_t extent[4]; };
struct Edge { uint32_t src_op, dst_op; DimMap map[4]; };
struct Cfg { uint8_t deg[4]; uint16_t dev_offset; uint16_t dev_stride; };
struct Machine { uint32_t n_nodes, gpus_per_node, intra_Bpns, inter_Bpns, intra_lat_ns, inter_lat_ns, elem_bytes; };
static_assert(sizeof(DimMap) == 12 && sizeof(Op) == 20 && sizeof(Edge) == 56 && sizeof(Cfg) == 8, "layout");

constexpr uint64_t INVALID = ~0ull;
constexpr uint32_t MAX_PARTS = 64;

struct TaskGraph {
    std::vector<uint64_t> exe;               // exeTime
    std::vector<uint32_t> dev;               // device row (compute device or link device)
    std::vector<std::vector<uint32_t>> out;  // O(t)
    std::vector<uint32_t> n_in;              // |I(t)|
    uint32_t n_compute = 0;
    uint32_t n_rows = 0;                     // number of device rows
    void add_dep(uint32_t a, uint32_t b) { out[a].push_back(b); n_in[b]++; }
    uint32_t add_task(uint64_t e, uint32_t d) {
        exe.push_back(e); dev.push_back(d); out.emplace_back(); n_in.push_back(0);
        return (uint32_t)exe.size() - 1;
    }
};

struct Box { int64_t lo[4], hi[4]; };

// Section 4: |c_i| = product of degrees; equal-size partitions (balanced floor split).
uint32_t parts_of(const Cfg& c) { return (uint32_t)c.deg[0] * c.deg[1] * c.deg[2] * c.deg[3]; }

bool cfg_valid(const Op& op, const Cfg& c, uint32_t n_dev, uint32_t max_parts) {
    for (int d = 0; d < 4; d++) {
        if (c.deg[d] < 1) return false;
        if (d >= op.ndim || !((op.par_mask >> d) & 1)) { if (c.deg[d] != 1) return false; }
        else if (c.deg[d] > op.extent[d]) return false;
    }
    if (parts_of(c) > max_parts) return false;
    return c.dev_offset < n_dev;
}

// output box of part k (row-major over the degree tuple, dim 0 slowest)
Box part_box(const Op& op, const Cfg& c, uint32_t k) {
    Box b;
    uint32_t idx[4], rem = k;
    for (int d = 3; d >= 0; d--) { idx[d] = rem % c.deg[d]; rem /= c.deg[d]; }
    for (int d = 0; d < 4; d++) {
        int64_t E = d < op.ndim ? op.extent[d] : 1;
        b.lo[d] = (int64_t)idx[d] * E / c.deg[d];
        b.hi[d] = (int64_t)(idx[d] + 1) * E / c.deg[d];
    }
    return b;
}

// The sub-tensor two tasks share through an edge, in elements (0: none).
// A reading edge (kind 0, the forward pass): map[d] belongs to dim d of the PRODUCER's tensor; the consumer
// part with box `cb` reads the range [cb.lo*stride + a, (cb.hi-1)*stride + b + 1) of it (along the consumer
// dim src_dim; the whole extent if src_dim < 0), clamped to the tensor; shared = what of that lies in the
// producer part's box `pb`.
// A contributing edge (kind 1, gradients flowing back along a forward edge): the same map with the roles
// exchanged.  map[d] belongs to dim d of the CONSUMER's tensor; the producer part with box `pb` contributes to
// the range [pb.lo*stride + a, (pb.hi-1)*stride + b + 1) of it (along the producer dim src_dim); shared =
// what of that lies in the consumer part's box `cb`.  The pairs and sizes are those of the forward edge,
// transposed.
uint64_t shared_elems(const Op& prod, const Op& cons, const Edge& e, const Box& pb, const Box& cb) {
    const bool contributes = e.map[0].kind != 0;
    const Op& space = contributes ? cons : prod;          // the tensor the ranges are taken in
    const Box& driving = contributes ? pb : cb;           // the part whose box goes through the map
    const Box& owning = contributes ? cb : pb;            // the part that holds a box of `space`
    uint64_t elems = 1;
    for (int d = 0; d < space.ndim; d++) {
        const DimMap& m = e.map[d];
        int64_t need_lo = 0, need_hi = space.extent[d];
        if (m.src_dim >= 0) {
            need_lo = driving.lo[m.src_dim] * (int64_t)m.stride + m.a;
            need_hi = (driving.hi[m.src_dim] - 1) * (int64_t)m.stride + m.b + 1;
            need_lo = std::max<int64_t>(need_lo, 0);
            need_hi = std::min<int64_t>(need_hi, space.extent[d]);
        }
        int64_t lo = std::max(need_lo, owning.lo[d]), hi = std::min(need_hi, owning.hi[d]);
        if (hi <= lo) return 0;
        elems *= (uint64_t)(hi - lo);
    }
    return elems;
}

// Section 5.1: the communication device that connects the two devices (see the readings: one link per
// ordered GPU pair inside a node, one per ordered node pair between nodes)
uint32_t link_row(const Machine& m, uint32_t from, uint32_t to) {
    uint32_t G = m.gpus_per_node, N = m.n_nodes, D = N * G;
    uint32_t na = from / G, nb = to / G;
    if (na == nb) return D + na * G * G + (from % G) * G + (to % G);
    return D + N * G * G + na * N + nb;
}

// Where the exeTime of a compute task comes from (Section 5.1 step 1): a table indexed by the
// op's number of parts, or a list per op keyed by the whole degree tuple (how long a task runs
// depends on which dims are split).
struct CostModel {
    const uint32_t* table; uint32_t n_cols;                           // [n_ops][n_cols], column parts-1
    const uint32_t* tuple_ptr; const uint32_t* tuples; const uint32_t* tuple_ns;   // or: op i's entries tuple_ptr[i]..tuple_ptr[i+1]
};

// false: the model has no time for this configuration
bool exe_time(const CostModel& cm, uint32_t i, const Cfg& c, uint32_t parts, uint64_t* out) {
    if (cm.table) { *out = cm.table[(size_t)i * cm.n_cols + (parts - 1)]; return true; }
    const uint32_t key = (uint32_t)c.deg[0] | ((uint32_t)c.deg[1] << 8) | ((uint32_t)c.deg[2] << 16) | ((uint32_t)c.deg[3] << 24);
    for (uint32_t t = cm.tuple_ptr[i]; t < cm.tuple_ptr[i + 1]; t++)
        if (cm.tuples[t] == key) { *out = cm.tuple_ns[t]; return true; }
    return false;
}

// Optional refinements of the inputs (all null = the plain forms):
// link_bw / link_lat [G][G]: bandwidth and latency of the link from local GPU a to local GPU b
// of one node (the same in every node; the diagonal is not used) instead of the machine's
// single intra-node figures -- the device topology's connections need not be alike.
// node_bw / node_lat [N][N]: bandwidth and latency of the network link from node a to node b (the
// diagonal is not used) instead of the machine's single inter-node figures.
// leader [n_ops]: tied configurations.  Section 4 gives every OPERATION one configuration; in a training
// iteration an operation appears as several ops of the graph (its forward and its backward computation;
// the unrolled steps of a recurrent layer that share parameters).  Op i then takes the configuration the
// strategy holds for op leader[i] (leader[leader[i]] == leader[i]); the strategy's entries for other ops
// are not read.  The configuration must be valid for every op that takes it.
// devmap [n_ops][64]: the device of every task given one by one (Section 4: a configuration
// assigns each task its device), instead of offset + k * stride.
// param_bytes / param_dims [n_ops]: parameter synchronisation.  Section 8 discusses how strategies
// differ in the data they move to synchronise parameters among replicas; Section 5.1 gives no
// construction for it.  Reading taken here: op i holds param_bytes[i] bytes of parameters, indexed by
// the output dims in param_dims[i] (bit d); its configuration cuts them into one shard per index
// along those dims, and the parts that differ only in the other dims are replicas of a shard.  The
// replica with index 0 in all other dims owns the shard; every other replica, when its task has
// finished, sends its gradient of the shard (ceil(param_bytes / shards) bytes) to the owner's
// device: one communication task per replica on another device than the owner, with the
// replica's compute task as its only predecessor and no successor.  The update itself and the
// way back are not modelled.  These tasks are created right after the communication tasks of
// the op's out-edges (so ids go op by op).
struct Extras {
    const uint32_t* link_bw; const uint32_t* link_lat; const uint16_t* devmap;
    const uint32_t* param_bytes; const uint8_t* param_dims;
    const uint32_t* node_bw; const uint32_t* node_lat;
    const uint32_t* leader;
};

uint64_t transfer_ns(const Machine& m, const Extras& x, uint32_t from, uint32_t to, uint64_t bytes) {
    const uint32_t G = m.gpus_per_node;
    const bool same_node = from / G == to / G;
    uint64_t bw = same_node ? m.intra_Bpns : m.inter_Bpns;
    uint64_t lat = same_node ? m.intra_lat_ns : m.inter_lat_ns;
    if (same_node && x.link_bw) {
        const size_t pair = (size_t)(from % G) * G + to % G;
        bw = x.link_bw[pair];
        lat = x.link_lat[pair];
    }
    if (!same_node && x.node_bw) {
        const size_t pair = (size_t)(from / G) * m.n_nodes + to / G;
        bw = x.node_bw[pair];
        lat = x.node_lat[pair];
    }
    return (bytes + bw - 1) / bw + lat;       // assumption A2, rounded up, plus the link's latency
}

// The readings above need the edge list producer by producer; ops in topological order.
bool graph_ok(uint32_t n_ops, uint32_t n_edges, const Edge* edges) {
    for (uint32_t e = 0; e < n_edges; e++) {
        if (edges[e].src_op >= n_ops || edges[e].dst_op >= n_ops || edges[e].src_op >= edges[e].dst_op) return false;
        if (e > 0 && edges[e - 1].src_op > edges[e].src_op) return false;
        for (int d = 1; d < 4; d++)
            if ((edges[e].map[d].kind != 0) != (edges[e].map[0].kind != 0)) return false;   // one kind per edge
    }
    return true;
}

bool build(uint32_t n_ops, const Op* ops, uint32_t n_edges, const Edge* edges, const Machine& m,
           const CostModel& cm, const Cfg* cfg, const Extras& x, TaskGraph& tg) {
    if (!graph_ok(n_ops, n_edges, edges)) return false;
    const uint32_t G = m.gpus_per_node, N = m.n_nodes, D = N * G;
    const uint32_t max_parts = cm.table ? std::min(MAX_PARTS, cm.n_cols) : MAX_PARTS;
    tg.n_rows = D + N * G * G + N * N;
    std::vector<uint32_t> first(n_ops), np(n_ops);
    // step 1: compute tasks t_{i:1..|c_i|}
    std::vector<Cfg> tied;
    if (x.leader) {
        tied.resize(n_ops);
        for (uint32_t i = 0; i < n_ops; i++) {
            if (x.leader[i] >= n_ops || x.leader[x.leader[i]] != x.leader[i]) return false;
            tied[i] = cfg[x.leader[i]];
        }
        cfg = tied.data();
    }
    for (uint32_t i = 0; i < n_ops; i++) {
        Cfg c = cfg[i];
        if (x.devmap) { c.dev_offset = 0; c.dev_stride = 1; }     // not used with explicit devices
        if (!cfg_valid(ops[i], c, D, max_parts)) return false;
        np[i] = parts_of(cfg[i]);
        uint64_t exe = 0;
        if (!exe_time(cm, i, cfg[i], np[i], &exe)) return false;
        first[i] = (uint32_t)tg.exe.size();
        for (uint32_t k = 0; k < np[i]; k++) {
            uint32_t dev = (uint32_t)((cfg[i].dev_offset + (uint64_t)k * cfg[i].dev_stride) % D);
            if (x.devmap) {
                dev = x.devmap[(size_t)i * MAX_PARTS + k];
                if (dev >= D) return false;
            }
            tg.add_task(exe, dev);
        }
    }
    tg.n_compute = (uint32_t)tg.exe.size();
    // step 2, op by op: per tensor edge out of the op, per pair of tasks with a shared sub-tensor
    std::vector<std::vector<uint32_t>> out_edges(n_ops);      // per producer, in the given order
    for (uint32_t e = 0; e < n_edges; e++) out_edges[edges[e].src_op].push_back(e);
    for (uint32_t i = 0; i < n_ops; i++) {
        for (uint32_t e : out_edges[i]) {
            const uint32_t j = edges[e].dst_op;
            for (uint32_t kp = 0; kp < np[i]; kp++) {
                Box pb = part_box(ops[i], cfg[i], kp);
                for (uint32_t kc = 0; kc < np[j]; kc++) {
                    Box cb = part_box(ops[j], cfg[j], kc);
                    uint64_t elems = shared_elems(ops[i], ops[j], edges[e], pb, cb);
                    if (!elems) continue;
                    uint32_t tp = first[i] + kp, tc = first[j] + kc;
                    if (tg.dev[tp] == tg.dev[tc]) { tg.add_dep(tp, tc); continue; }
                    uint32_t c = tg.add_task(transfer_ns(m, x, tg.dev[tp], tg.dev[tc], elems * m.elem_bytes),
                                             link_row(m, tg.dev[tp], tg.dev[tc]));
                    tg.add_dep(tp, c);
                    tg.add_dep(c, tc);
                }
            }
        }
        // parameter synchronisation of the op (see Extras)
        if (x.param_bytes && x.param_bytes[i]) {
            const Cfg& c = cfg[i];
            uint32_t shards = 1;
            for (int d = 0; d < 4; d++) if ((x.param_dims[i] >> d) & 1) shards *= c.deg[d];
            const uint64_t shard_bytes = ((uint64_t)x.param_bytes[i] + shards - 1) / shards;
            for (uint32_t k = 0; k < np[i]; k++) {
                // index of part k along each dim (dim 0 slowest), and the owner: the same index
                // along the parameter dims, 0 along the others
                uint32_t idx[4], rem = k;
                for (int d = 3; d >= 0; d--) { idx[d] = rem % c.deg[d]; rem /= c.deg[d]; }
                uint32_t owner = 0;
                for (int d = 0; d < 4; d++) owner = owner * c.deg[d] + (((x.param_dims[i] >> d) & 1) ? idx[d] : 0);
                const uint32_t tk = first[i] + k, to = first[i] + owner;
                if (owner == k || tg.dev[tk] == tg.dev[to]) continue;
                uint32_t t = tg.add_task(transfer_ns(m, x, tg.dev[tk], tg.dev[to], shard_bytes), link_row(m, tg.dev[tk], tg.dev[to]));
                tg.add_dep(tk, t);
            }
        }
    }
    return true;
}

// Section 5.2, full simulation.  Every task is NOTREADY until its last predecessor is COMPLETE; then it
// is READY, and its readyTime is the largest endTime among its predecessors (0 for a task without
// any).  READY tasks wait in one global queue ordered by (readyTime, task id).  The task at the head
// of the queue is assigned to its device: the device runs one task at a time, in the order the
// tasks are handed to it, so the task starts when both its inputs and the device are available
// (assumptions A3, A4) and ends exeTime later.  The result is the largest endTime.
// ready_o / start_o / end_o (may be null) receive the timeline.
enum TaskState : uint8_t { NOTREADY, READY, COMPLETE };

uint64_t simulate(const TaskGraph& tg, uint64_t* ready_o, uint64_t* start_o, uint64_t* end_o) {
    const size_t n = tg.exe.size();
    std::vector<uint64_t> ready_time(n, 0), start_time(n, 0), end_time(n, 0);
    std::vector<TaskState> state(n, NOTREADY);
    std::vector<uint32_t> complete_preds(n, 0);          // predecessors of the task that are COMPLETE
    std::vector<uint64_t> device_busy_until(tg.n_rows, 0);
    std::set<std::pair<uint64_t, uint32_t>> ready_queue;   // (readyTime, id) of every READY task, ascending

    for (uint32_t t = 0; t < n; t++)
        if (tg.n_in[t] == 0) { state[t] = READY; ready_queue.emplace(0, t); }

    uint64_t makespan = 0;
    while (!ready_queue.empty()) {
        const uint32_t t = ready_queue.begin()->second;
        ready_queue.erase(ready_queue.begin());
        uint64_t& busy_until = device_busy_until[tg.dev[t]];
        start_time[t] = std::max(ready_time[t], busy_until);
        end_time[t] = start_time[t] + tg.exe[t];
        busy_until = end_time[t];
        state[t] = COMPLETE;
        makespan = std::max(makespan, end_time[t]);
        for (uint32_t succ : tg.out[t]) {
            ready_time[succ] = std::max(ready_time[succ], end_time[t]);
            if (++complete_preds[succ] == tg.n_in[succ]) {
                state[succ] = READY;
                ready_queue.emplace(ready_time[succ], succ);
            }
        }
    }
    if (ready_o) std::memcpy(ready_o, ready_time.data(), n * 8);
    if (start_o) std::memcpy(start_o, start_time.data(), n * 8);
    if (end_o) std::memcpy(end_o, end_time.data(), n * 8);
    return makespan;
}

}  // namespace

extern "C" {

// 1 if the edge list is one the oracle accepts (see graph_ok), else 0
int ffo_graph_ok(uint32_t n_ops, uint32_t n_edges, const void* edges) { return graph_ok(n_ops, n_edges, (const Edge*)edges) ? 1 : 0; }

// Build the task graph of one strategy.  Returns an opaque handle or null if the strategy
// is invalid.
// cost / n_cols: the table by number of parts; or cost = null and the three tuple arrays.
void* ffo_build(uint32_t n_ops, const void* ops, uint32_t n_edges, const void* edges, const void* machine,
                const uint32_t* cost, uint32_t n_cols, const uint32_t* tuple_ptr, const uint32_t* tuples,
                const uint32_t* tuple_ns, const void* cfg, const uint32_t* link_bw, const uint32_t* link_lat,
                const uint16_t* devmap, const uint32_t* param_bytes, const uint8_t* param_dims,
                const uint32_t* node_bw, const uint32_t* node_lat, const uint32_t* leader) {
    TaskGraph* tg = new TaskGraph;
    const CostModel cm{cost, n_cols, tuple_ptr, tuples, tuple_ns};
    const Extras x{link_bw, link_lat, devmap, param_bytes, param_dims, node_bw, node_lat, leader};
    if (!build(n_ops, (const Op*)ops, n_edges, (const Edge*)edges, *(const Machine*)machine, cm,
               (const Cfg*)cfg, x, *tg)) { delete tg; return nullptr; }
    return tg;
}

// A task graph given directly (for pins on hand-made graphs): deps are (src, dst) pairs.
void* ffo_from_arrays(uint32_t n_tasks, const uint64_t* exe, const uint32_t* dev, uint32_t n_rows,
                      uint32_t n_deps, const uint32_t* dep_src, const uint32_t* dep_dst) {
    TaskGraph* tg = new TaskGraph;
    for (uint32_t t = 0; t < n_tasks; t++) tg->add_task(exe[t], dev[t]);
    tg->n_compute = n_tasks;
    tg->n_rows = n_rows;
    for (uint32_t k = 0; k < n_deps; k++) tg->add_dep(dep_src[k], dep_dst[k]);
    return tg;
}

void ffo_counts(const void* h, uint32_t* n_tasks, uint32_t* n_compute, uint32_t* n_deps, uint32_t* n_rows) {
    const TaskGraph* tg = (const TaskGraph*)h;
    uint32_t nd = 0;
    for (auto& o : tg->out) nd += (uint32_t)o.size();
    *n_tasks = (uint32_t)tg->exe.size(); *n_compute = tg->n_compute; *n_deps = nd; *n_rows = tg->n_rows;
}

void ffo_export(const void* h, uint64_t* exe, uint32_t* dev, uint32_t* dep_src, uint32_t* dep_dst) {
    const TaskGraph* tg = (const TaskGraph*)h;
    size_t k = 0;
    for (size_t t = 0; t < tg->exe.size(); t++) {
        exe[t] = tg->exe[t]; dev[t] = tg->dev[t];
        for (uint32_t s : tg->out[t]) { dep_src[k] = (uint32_t)t; dep_dst[k] = s; k++; }
    }
}

uint64_t ffo_simulate(const void* h, uint64_t* ready, uint64_t* start, uint64_t* end) {
    return simulate(*(const TaskGraph*)h, ready, start, end);
}

void ffo_free(void* h) { delete (TaskGraph*)h; }

// build + simulate for B strategies ([B][n_ops] configs); invalid strategy -> all-ones.
// n_threads > 1 splits the candidates statically over threads (one independent oracle run each).
void ffo_batch(uint32_t n_ops, const void* ops, uint32_t n_edges, const void* edges, const void* machine,
               const uint32_t* cost, uint32_t n_cols, const uint32_t* tuple_ptr, const uint32_t* tuples,
               const uint32_t* tuple_ns, const void* cfgs, uint32_t B, uint64_t* out_ns, uint32_t n_threads,
               const uint32_t* link_bw, const uint32_t* link_lat, const uint16_t* devmaps, const uint32_t* param_bytes,
               const uint8_t* param_dims, const uint32_t* node_bw, const uint32_t* node_lat, const uint32_t* leader) {
    const CostModel cm{cost, n_cols, tuple_ptr, tuples, tuple_ns};
    auto work = [&](uint32_t b0, uint32_t b1) {
        for (uint32_t b = b0; b < b1; b++) {
            TaskGraph tg;
            const Extras x{link_bw, link_lat, devmaps ? devmaps + (size_t)b * n_ops * MAX_PARTS : nullptr, param_bytes, param_dims,
                           node_bw, node_lat, leader};
            bool ok = build(n_ops, (const Op*)ops, n_edges, (const Edge*)edges, *(const Machine*)machine, cm,
                            (const Cfg*)cfgs + (size_t)b * n_ops, x, tg);
            out_ns[b] = ok ? simulate(tg, nullptr, nullptr, nullptr) : INVALID;
        }
    };
    if (n_threads <= 1) { work(0, B); return; }
    std::vector<std::thread> th;
    for (uint32_t t = 0; t < n_threads; t++)
        th.emplace_back(work, (uint32_t)((uint64_t)B * t / n_threads), (uint32_t)((uint64_t)B * (t + 1) / n_threads));
    for (auto& t : th) t.join();
}

}  // extern "C"
