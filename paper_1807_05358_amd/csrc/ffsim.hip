// Host side of the C boundary declared in include/ff_sim.h: validation, upload of the
// constant tables, workspace bookkeeping and kernel launches.  No torch types here.
#include "../../include/ff_sim.h"
#include <chrono>

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <new>
#include <vector>

#include "ffsim_select.h"
#include "ffsim_sweep.h"

using namespace ffsim;

namespace {

template <typename T>
int upload(const std::vector<T>& v, T** out) {
    *out = nullptr;
    size_t bytes = std::max<size_t>(v.size(), 1) * sizeof(T);
    if (hipMalloc((void**)out, bytes) != hipSuccess) return FF_ENOMEM;
    if (!v.empty() && hipMemcpy(*out, v.data(), v.size() * sizeof(T), hipMemcpyHostToDevice) != hipSuccess) return FF_EHIP;
    return FF_OK;
}

uint32_t magic_plus1(uint32_t d) { return d <= 1 ? 0u : (uint32_t)((1ull << 32) / d) + 1u; }
uint32_t magic_floor(uint32_t d) { return d <= 1 ? 0xffffffffu : (uint32_t)((1ull << 32) / d); }

}  // namespace

struct ff_sim {
    SimDev dev{};
    DOp* d_ops = nullptr;
    DEdge* d_edges = nullptr;
    DEdge* d_in_edges = nullptr;
    uint32_t* d_cost = nullptr;
    uint32_t* d_magic = nullptr;
    bool wide = false;            // some tensor has 2^32 bytes or more, or a link row's running sum may pass 2^32 ns
    bool big_tensors = false;     // some tensor has 2^32 bytes or more
    ff_machine_t mach{};
    uint32_t links_gen = 0;       // counts ff_sim_set_links / ff_sim_set_params calls (a chain set's stored timelines depend on both)
    std::vector<DOp> h_ops;       // host copy of the op records (ff_sim_set_params rewrites two fields)
    std::vector<uint32_t> intra_bw, intra_lat, node_bw, node_lat;   // the link tables in force (empty: the machine's single figures)
    std::vector<uint32_t> ties;   // per op the op whose configuration it takes (empty: its own)
    bool has_contributing = false;   // the graph has contributing (gradient) edges: served by the kernels with the refinements
    bool lds_words = false;       // task words of a candidate fit in LDS (small graphs)
    size_t slot_bytes = 0;        // HBM scratch per resident wavefront (also used by chains)
    // the batch kernel may keep the per-edge set-up of a candidate (all extents must fit 16 bits):
    // behind the task words, in the HBM slot, or in LDS for graphs whose words live there
    bool cache_ok = false;
    bool chain_cache = false;     // the same for chains: only the extents matter, the set-up lives in the chain's memory
    size_t batch_slot_bytes = 0;  // slot_bytes, plus the kept set-up where it lives in HBM
    size_t lds_cached = 0;        // dynamic LDS of the caching variant (= lds if the set-up lives in HBM)
    uint32_t max_slots_cached = 0;
    size_t lds = 0;               // dynamic LDS per wavefront, batch kernel
    size_t lds_common = 0;        // device rows + queue levels 1 and 2
    size_t lds_chain = 0;         // dynamic LDS per wavefront, chain kernel (adds the strategy; words in HBM)
    uint32_t max_slots = 0;       // wavefronts the device can hold at once (batch kernel)
    uint32_t max_try_slots = 0;   // same for the trial-mutation kernel
    void* ws = nullptr;
    size_t ws_bytes = 0;
    ff_stats_t* d_stats = nullptr;
};

struct ff_chains {
    ff_sim* sim = nullptr;
    uint32_t C = 0;
    uint32_t n_snaps = 0;
    size_t stride = 0;             // bytes per chain
    unsigned char* d_mem = nullptr; // [C] chain blocks: strategy, task words, endTimes, snapshots
    uint32_t* d_flags = nullptr;   // [C] nonzero once a chain saw an out-of-range mutation
    uint32_t* d_counter = nullptr; // work counter of the trial-mutation kernel
    uint32_t links_gen = 0;        // sim->links_gen when the chains were created
    const uint32_t* checked_ptr = nullptr;   // the proposal ranges ff_sim_search has checked last
    uint32_t checked_n = 0;
    // ff_sim_search_ahead: proposals [K][C], their simulated times [K][C], steps done per chain [C]; K <= ahead_cap
    uint32_t* d_ahead_muts = nullptr;
    uint64_t* d_ahead_ns = nullptr;
    uint32_t* d_ahead_done = nullptr;
    uint32_t ahead_cap = 0;
};

// Scratch of ff_sim_neighbours_noalloc: the index of every op's first neighbour (one entry per op of the
// range plus the total) and a status word, in device memory that exists from the moment the library is
// loaded, so that the call allocates nothing.  Every GPU holds its own copy at its own address; in host
// code the array's name is only a handle for hipGetSymbolAddress, never an address to hand to a kernel.
constexpr uint32_t NEIGHBOUR_SCRATCH_OPS = FF_MAX_OPS;
static __device__ __align__(256) uint32_t neighbour_scratch[NEIGHBOUR_SCRATCH_OPS + 1 + 63];
constexpr int SCRATCH_MAX_GPUS = 64;
static uint32_t* neighbour_scratch_ptr[SCRATCH_MAX_GPUS];      // per device, resolved once

// the current device's copy of the scratch array, or null if it cannot be resolved
static uint32_t* neighbour_scratch_of_current_device() {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= SCRATCH_MAX_GPUS) return nullptr;
    if (!neighbour_scratch_ptr[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(neighbour_scratch)) != hipSuccess) return nullptr;
        neighbour_scratch_ptr[dev] = (uint32_t*)p;
    }
    return neighbour_scratch_ptr[dev];
}

static bool batch_cached(const ff_sim* s, uint32_t B);
static uint32_t batch_slots(const ff_sim* s, uint32_t B);

constexpr uint32_t CHAIN_SNAPSHOTS = 32;
static_assert(CHAIN_SNAPSHOTS <= MAX_SNAPSHOTS, "one bit per snapshot in ChainMeta::loc");

static KernelChoice choice(const ff_sim* s, bool cache) {
    return KernelChoice{s->wide, s->lds_words, s->d_stats != nullptr, cache, s->dev.n_ops, s->dev.n_groups, s->dev.max_parts};
}
// ext: which refinements the launch needs (0 none; 1 link tables, explicit devices, parameter traffic; 2 also
// contributing edges or tied configurations).  Machines with four GPUs per node (all benchmark configurations)
// have kernels compiled for that node size.
static int ext_level(const ff_sim* s, bool devmaps = false) {
    if (s->dev.ties || s->has_contributing) return 2;
    return (s->dev.link_table || s->dev.node_table || s->dev.sync || devmaps) ? 1 : 0;
}
static batch_kernel_t batch_kernel(const ff_sim* s, bool cached, int ext = 0) {
    const KernelChoice k = choice(s, cached);
    if (s->dev.gpus_per_node == 4) return ext == 2 ? batch_kernels<2, 4>(k) : (ext == 1 ? batch_kernels<1, 4>(k) : batch_kernels<0, 4>(k));
    return ext == 2 ? batch_kernels<2, 0>(k) : (ext == 1 ? batch_kernels<1, 0>(k) : batch_kernels<0, 0>(k));
}
// chains keep the per-edge set-up in their own memory whenever the extents allow it
static chain_kernel_t chain_kernel(const ff_sim* s) {
    const KernelChoice k = choice(s, s->chain_cache);
    const int ext = ext_level(s);
    if (s->dev.gpus_per_node == 4) return ext == 2 ? chain_kernels<2, 4>(k) : (ext == 1 ? chain_kernels<1, 4>(k) : chain_kernels<0, 4>(k));
    return ext == 2 ? chain_kernels<2, 0>(k) : (ext == 1 ? chain_kernels<1, 0>(k) : chain_kernels<0, 0>(k));
}
static try_kernel_t try_kernel(const ff_sim* s) {
    const KernelChoice k = choice(s, s->chain_cache);
    const int ext = ext_level(s);
    if (s->dev.gpus_per_node == 4) return ext == 2 ? try_kernels<2, 4>(k) : (ext == 1 ? try_kernels<1, 4>(k) : try_kernels<0, 4>(k));
    return ext == 2 ? try_kernels<2, 0>(k) : (ext == 1 ? try_kernels<1, 0>(k) : try_kernels<0, 0>(k));
}

// A launch with more than 64 KB of dynamic LDS (gfx950 allows a workgroup up to 160 KB) has to be
// announced for the kernel first.
static bool allow_lds(const void* kernel, size_t bytes) {
    if (bytes <= 64 * 1024) return true;
    return hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes) == hipSuccess;
}

static void release(ff_sim* s) {
    if (!s) return;
    hipFree(s->d_ops); hipFree(s->d_edges); hipFree(s->d_in_edges); hipFree(s->d_cost); hipFree(s->d_magic);
    delete s;
}

extern "C" {

const char* ff_sim_strerror(int code) {
    switch (code) {
        case FF_OK: return "ok";
        case FF_EINVAL: return "invalid argument";
        case FF_ENOMEM: return "out of memory";
        case FF_EWORKSPACE: return "workspace missing or too small";
        case FF_ERANGE: return "size limit exceeded";
        case FF_EHIP: return "HIP runtime error";
        default: return "unknown error";
    }
}

}  // extern "C"

// cost: the device image of the cost model.  n_cols >= 1: the table [n_ops][n_cols] indexed by the
// number of parts.  n_cols == 0: costs keyed by the degree tuple, packed as ptr[n_ops+1], then the
// tuples of all ops, then their exeTimes.
// the constants buffer of the kernels (layout: LINK_TABLE_AT in ffsim_device.h)
// intra: per ordered pair of local GPUs (G*G entries) or empty; inter: per ordered pair of nodes (N*N) or empty
// (an area that is not given is filled with the machine's single figures; it is then not read); ties: per op the
// op whose configuration it takes, or empty.  Layout: ffsim_device.h.
static std::vector<uint32_t> constants_image(const ff_machine_t& m, const std::vector<uint32_t>& intra_bw, const std::vector<uint32_t>& intra_lat,
                                             const std::vector<uint32_t>& node_bw, const std::vector<uint32_t>& node_lat,
                                             const std::vector<uint32_t>& ties) {
    const size_t G2 = (size_t)m.gpus_per_node * m.gpus_per_node, N2 = (size_t)m.n_nodes * m.n_nodes;
    const size_t tie_at = tie_table_at(m.gpus_per_node, m.n_nodes);
    std::vector<uint32_t> c(tie_at + std::max<size_t>(ties.size(), 1), 0);
    for (uint32_t d = 2; d <= 64; d++) c[d] = magic_plus1(d);
    for (size_t p = 0; p < G2; p++) {
        const uint32_t bw = intra_bw.empty() ? m.intra_Bpns : intra_bw[p];
        c[LINK_TABLE_AT + 4 * p + 0] = bw;
        c[LINK_TABLE_AT + 4 * p + 1] = magic_floor(bw);
        c[LINK_TABLE_AT + 4 * p + 2] = intra_bw.empty() ? m.intra_lat_ns : intra_lat[p];
    }
    for (size_t p = 0; p < N2; p++) {
        const uint32_t bw = node_bw.empty() ? m.inter_Bpns : node_bw[p];
        c[LINK_TABLE_AT + 4 * (G2 + p) + 0] = bw;
        c[LINK_TABLE_AT + 4 * (G2 + p) + 1] = magic_floor(bw);
        c[LINK_TABLE_AT + 4 * (G2 + p) + 2] = node_bw.empty() ? m.inter_lat_ns : node_lat[p];
    }
    std::copy(ties.begin(), ties.end(), c.begin() + tie_at);
    return c;
}

// The narrow kernels count elements, bytes and a link row's running sum of transfer times in
// 32 bits: every tensor must stay below 2^32 bytes, and gpus_per_node of the longest possible
// transfers (the most one producer part can queue on one row) below 2^32 ns.  Everything else
// runs in the 64-bit (WIDE) kernels.
static bool needs_wide(bool big_tensors, uint32_t bw_min, uint32_t lat_max, uint32_t gpus_per_node) {
    const uint64_t ns_max = (0xffffffffull + bw_min - 1) / bw_min + lat_max;
    return big_tensors || ns_max * gpus_per_node >= (1ull << 32);
}

static int create_impl(const ff_opgraph_t* g, const ff_machine_t* m, std::vector<uint32_t>& cost, uint32_t n_cols, ff_sim_t** out) {
    if (g->n_ops > FF_MAX_OPS) return FF_ERANGE;
    if (m->n_nodes < 1 || m->gpus_per_node < 1 || m->intra_Bpns < 1 || m->inter_Bpns < 1 || m->elem_bytes < 1) return FF_EINVAL;
    const uint64_t D = (uint64_t)m->n_nodes * m->gpus_per_node;
    if (D > FF_MAX_DEVICES) return FF_ERANGE;
    const uint64_t n_rows = D + (uint64_t)m->n_nodes * m->gpus_per_node * m->gpus_per_node + (uint64_t)m->n_nodes * m->n_nodes;

    std::vector<DOp> ops(g->n_ops);
    unsigned __int128 max_bytes = 0;
    uint32_t max_extent = 1;
    for (uint32_t i = 0; i < g->n_ops; i++) {
        const ff_op_t& o = g->ops[i];
        if (o.ndim < 1 || o.ndim > FF_MAX_DIMS) return FF_EINVAL;
        unsigned __int128 elems = 1;
        for (int d = 0; d < 4; d++) {
            uint32_t e = d < o.ndim ? o.extent[d] : 1;
            if (e < 1) return FF_EINVAL;
            if (e > FF_MAX_EXTENT) return FF_ERANGE;
            ops[i].extent[d] = e;
            max_extent = std::max(max_extent, e);
            elems *= e;
        }
        max_bytes = std::max(max_bytes, elems * m->elem_bytes);
        ops[i].ndim = o.ndim;
        ops[i].par_mask = o.par_mask & ((1u << o.ndim) - 1);
        ops[i].out_begin = ops[i].out_end = 0;
    }
    if (max_bytes >= ((unsigned __int128)1 << 62)) return FF_ERANGE;

    std::vector<DEdge> edges(g->n_edges);
    std::vector<uint32_t> in_count(g->n_ops, 0);
    bool has_contributing = false;
    for (uint32_t k = 0; k < g->n_edges; k++) {
        const ff_edge_t& e = g->edges[k];
        if (e.src_op >= g->n_ops || e.dst_op >= g->n_ops || e.src_op >= e.dst_op) return FF_EINVAL;
        if (k > 0) {
            const ff_edge_t& p = g->edges[k - 1];
            if (p.src_op > e.src_op || (p.src_op == e.src_op && p.dst_op > e.dst_op)) return FF_EINVAL;
        }
        DEdge& de = edges[k];
        de.src = e.src_op;
        de.dst = e.dst_op;
        // a contributing edge exchanges the roles: the maps belong to the consumer's dims and name producer dims
        const bool contributes = e.map[0].kind != 0;
        for (int d = 0; d < 4; d++)
            if (e.map[d].kind > 1 || (e.map[d].kind != 0) != contributes) return FF_EINVAL;
        has_contributing = has_contributing || contributes;
        const uint32_t space_op = contributes ? e.dst_op : e.src_op, driving_op = contributes ? e.src_op : e.dst_op;
        de.src_ndim = ops[space_op].ndim;
        de.eid = k;
        de.kind = contributes ? 1u : 0u;
        de.unused[0] = de.unused[1] = de.unused[2] = 0;
        for (int d = 0; d < 4; d++) {
            de.src_extent[d] = ops[space_op].extent[d];
            DMap& dm = de.map[d];
            const ff_dimmap_t& sm = e.map[d];
            if (d >= g->ops[space_op].ndim || sm.src_dim < 0) { dm = DMap{-1, 1, 0, 0, 1}; continue; }
            if (sm.src_dim >= g->ops[driving_op].ndim || sm.stride < 1) return FF_EINVAL;
            if (sm.stride > FF_MAX_MAP_STRIDE || sm.a > FF_MAX_MAP_OFFSET || sm.a < -FF_MAX_MAP_OFFSET ||
                sm.b > FF_MAX_MAP_OFFSET || sm.b < -FF_MAX_MAP_OFFSET) return FF_ERANGE;
            dm = DMap{sm.src_dim, sm.stride, sm.a, sm.b, ops[driving_op].extent[sm.src_dim]};
        }
        in_count[e.dst_op]++;
    }
    // out-edges of an op are a contiguous range (edges are sorted by producer); in-edges are a
    // second copy of the records grouped by consumer
    {
        uint32_t k = 0;
        for (uint32_t i = 0; i < g->n_ops; i++) {
            ops[i].out_begin = k;
            while (k < g->n_edges && edges[k].src == i) k++;
            ops[i].out_end = k;
            ops[i].param_bytes = ops[i].param_dims = 0;
            if (ops[i].out_end > ops[i].out_begin) ops[i].first = edges[ops[i].out_begin];
            else std::memset(&ops[i].first, 0, sizeof(DEdge));
        }
    }
    std::vector<DEdge> in_edges(g->n_edges);
    {
        uint32_t acc = 0;
        for (uint32_t i = 0; i < g->n_ops; i++) {
            if (in_count[i] > FF_MAX_IN_EDGES) return FF_ERANGE;   // pending-input counter has 15 bits
            ops[i].in_begin = acc; acc += in_count[i]; ops[i].in_end = ops[i].in_begin;
        }
        for (uint32_t k = 0; k < g->n_edges; k++) in_edges[ops[edges[k].dst].in_end++] = edges[k];
    }
    std::vector<uint32_t> magic = constants_image(*m, {}, {}, {}, {}, {});

    ff_sim* s = new (std::nothrow) ff_sim;
    if (!s) return FF_ENOMEM;
    int rc;
    if ((rc = upload(ops, &s->d_ops)) || (rc = upload(edges, &s->d_edges)) || (rc = upload(in_edges, &s->d_in_edges)) ||
        (rc = upload(cost, &s->d_cost)) || (rc = upload(magic, &s->d_magic))) { release(s); return rc; }

    s->h_ops = ops;
    s->has_contributing = has_contributing;
    SimDev& S = s->dev;
    S.n_ops = g->n_ops; S.n_edges = g->n_edges; S.n_cols = n_cols;
    S.max_parts = n_cols ? std::min<uint32_t>(FF_MAX_PARTS, n_cols) : FF_MAX_PARTS;
    S.n_nodes = m->n_nodes; S.gpus_per_node = m->gpus_per_node; S.n_dev = (uint32_t)D; S.n_rows = (uint32_t)n_rows;
    S.bw_intra = m->intra_Bpns; S.bw_inter = m->inter_Bpns; S.lat_intra = m->intra_lat_ns; S.lat_inter = m->inter_lat_ns;
    S.elem_bytes = m->elem_bytes;
    S.m_bw_intra = magic_floor(m->intra_Bpns); S.m_bw_inter = magic_floor(m->inter_Bpns);
    S.magic_dev = magic_plus1((uint32_t)D); S.magic_gpn = magic_plus1(m->gpus_per_node);
    S.pass_dev = D == 1 ? 0xffffffffu : 0u; S.pass_gpn = m->gpus_per_node == 1 ? 0xffffffffu : 0u;
    S.n_ops_pad = (g->n_ops + 63) & ~63u;
    S.n_groups = S.n_ops_pad / 64;
    s->mach = *m;
    s->big_tensors = max_bytes >= ((unsigned __int128)1 << 32);
    s->wide = needs_wide(s->big_tensors, std::min(m->intra_Bpns, m->inter_Bpns), std::max(m->intra_lat_ns, m->inter_lat_ns),
                         m->gpus_per_node);
    s->slot_bytes = (slot_bytes(S.n_ops, S.n_ops_pad) + 255) & ~(size_t)255;
    s->lds_common = lds_common_bytes(S.n_rows, S.n_ops_pad);
    s->lds_chain = s->lds_common + (size_t)S.n_ops_pad * 8;
    int dev_id = 0, cus = 0, per_cu = 0, lds_limit = 0;
    if (hipGetDevice(&dev_id) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev_id) != hipSuccess ||
        hipDeviceGetAttribute(&lds_limit, hipDeviceAttributeMaxSharedMemoryPerBlock, dev_id) != hipSuccess) { release(s); return FF_EHIP; }
    // device rows, queue levels and (chains) the strategy of one candidate must fit a workgroup's LDS
    if (s->lds_chain > (size_t)lds_limit) { release(s); return FF_ERANGE; }
    // small graphs keep a candidate's task words in LDS, as long as four wavefronts (one per
    // SIMD) still fit in a CU's 160 KB
    const size_t lds_with_words = ((slot_bytes(S.n_ops, S.n_ops_pad) + 15) & ~(size_t)15) + s->lds_common;
#ifdef FFSIM_FORCE_HBM
    s->lds_words = false;
#else
    s->lds_words = lds_with_words <= 40 * 1024;
#endif
    s->lds = s->lds_words ? lds_with_words : s->lds_common;
    s->cache_ok = max_extent <= ECACHE_MAX_EXTENT && g->n_edges > 0;
    s->chain_cache = s->cache_ok;
    s->batch_slot_bytes = s->slot_bytes;
    s->lds_cached = s->lds;
    if (s->cache_ok) {
        if (s->lds_words) {
            s->lds_cached = lds_with_words + ecache_bytes(S.n_edges);
            if (s->lds_cached > 40 * 1024) s->cache_ok = false;
        } else {
            s->batch_slot_bytes = (((slot_bytes(S.n_ops, S.n_ops_pad) + 15) & ~(size_t)15) + ecache_bytes(S.n_edges) + 255) & ~(size_t)255;
        }
    }

    if (!allow_lds((const void*)batch_kernel(s, false), s->lds) || !allow_lds((const void*)try_kernel(s), s->lds_common) ||
        (s->cache_ok && !allow_lds((const void*)batch_kernel(s, true), s->lds_cached))) { release(s); return FF_EHIP; }
    hipError_t e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, batch_kernel(s, false), WAVE, s->lds);
    if (e != hipSuccess || per_cu < 1) per_cu = 1;
    s->max_slots = (uint32_t)cus * (uint32_t)per_cu;
    per_cu = 0;
    if (s->cache_ok) {
        e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, batch_kernel(s, true), WAVE, s->lds_cached);
        if (e != hipSuccess || per_cu < 1) per_cu = 1;
        s->max_slots_cached = (uint32_t)cus * (uint32_t)per_cu;
    }
    per_cu = 0;
    e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, try_kernel(s), WAVE, s->lds_common);
    if (e != hipSuccess || per_cu < 1) per_cu = 1;
    s->max_try_slots = (uint32_t)cus * (uint32_t)per_cu;
    // the address of this device's scratch array (ff_sim_neighbours_noalloc) is looked up here, once per device
    if (!neighbour_scratch_of_current_device()) { release(s); return FF_EHIP; }
    *out = s;
    return FF_OK;
}

extern "C" {

int ff_sim_create(const ff_opgraph_t* g, const ff_machine_t* m, const ff_costtable_t* ct, ff_sim_t** out) {
    if (!out) return FF_EINVAL;
    *out = nullptr;
    if (!g || !m || !ct || !g->ops || (g->n_edges && !g->edges) || !ct->ns) return FF_EINVAL;
    if (g->n_ops < 1 || ct->n_ops != g->n_ops || ct->n_cols < 1) return FF_EINVAL;
    std::vector<uint32_t> cost((size_t)g->n_ops * ct->n_cols);
    for (size_t k = 0; k < cost.size(); k++) {
        if (ct->ns[k] < 1) return FF_EINVAL;   // every exeTime >= 1
        cost[k] = ct->ns[k];
    }
    return create_impl(g, m, cost, ct->n_cols, out);
}

int ff_sim_create_tuplecost(const ff_opgraph_t* g, const ff_machine_t* m, const ff_tuplecost_t* tc, ff_sim_t** out) {
    if (!out) return FF_EINVAL;
    *out = nullptr;
    if (!g || !m || !tc || !g->ops || (g->n_edges && !g->edges) || !tc->tuple_ptr || !tc->tuples || !tc->ns) return FF_EINVAL;
    if (g->n_ops < 1 || tc->n_ops != g->n_ops || tc->tuple_ptr[0] != 0) return FF_EINVAL;
    const uint32_t E = tc->tuple_ptr[g->n_ops];
    if (E < 1 || E > (1u << 30)) return FF_ERANGE;
    for (uint32_t i = 0; i < g->n_ops; i++) {
        if (tc->tuple_ptr[i] > tc->tuple_ptr[i + 1] || tc->tuple_ptr[i + 1] > E) return FF_EINVAL;
        for (uint32_t t = tc->tuple_ptr[i]; t < tc->tuple_ptr[i + 1]; t++) {
            if (tc->ns[t] < 1) return FF_EINVAL;                                              // every exeTime >= 1
            if (t > tc->tuple_ptr[i] && tc->tuples[t - 1] >= tc->tuples[t]) return FF_EINVAL;   // ascending, no duplicates
        }
    }
    std::vector<uint32_t> cost;
    cost.reserve((size_t)g->n_ops + 1 + 2 * (size_t)E);
    cost.insert(cost.end(), tc->tuple_ptr, tc->tuple_ptr + g->n_ops + 1);
    cost.insert(cost.end(), tc->tuples, tc->tuples + E);
    cost.insert(cost.end(), tc->ns, tc->ns + E);
    return create_impl(g, m, cost, 0, out);
}

void ff_sim_destroy(ff_sim_t* s) { release(s); }

int ff_sim_set_params(ff_sim_t* s, const uint32_t* param_bytes, const uint8_t* param_dims) {
    if (!s || (param_bytes && !param_dims)) return FF_EINVAL;
    bool any = false;
    std::vector<DOp> ops = s->h_ops;
    for (uint32_t i = 0; i < s->dev.n_ops; i++) {
        DOp& o = ops[i];
        o.param_bytes = param_bytes ? param_bytes[i] : 0;
        o.param_dims = param_bytes ? (param_dims[i] & ((1u << o.ndim) - 1)) : 0;
        any = any || o.param_bytes;
    }
    if (hipDeviceSynchronize() != hipSuccess) return FF_EHIP;       // no launch may still read the old records
    if (hipMemcpy(s->d_ops, ops.data(), ops.size() * sizeof(DOp), hipMemcpyHostToDevice) != hipSuccess) return FF_EHIP;
    s->h_ops.swap(ops);
    s->dev.sync = any ? 1u : 0u;
    s->links_gen++;
    return FF_OK;
}

// uploads the constants for the link tables and ties in force and re-derives what depends on them
static int apply_link_tables(ff_sim_t* s) {
    const ff_machine_t& m = s->mach;
    const uint32_t G = m.gpus_per_node, N = m.n_nodes;
    uint32_t bw_min = 0xffffffffu, lat_max = 0;
    if (s->intra_bw.empty()) { bw_min = std::min(bw_min, m.intra_Bpns); lat_max = std::max(lat_max, m.intra_lat_ns); }
    else
        for (uint32_t a = 0; a < G; a++)
            for (uint32_t b = 0; b < G; b++)
                if (a != b) { bw_min = std::min(bw_min, s->intra_bw[a * G + b]); lat_max = std::max(lat_max, s->intra_lat[a * G + b]); }
    if (s->node_bw.empty()) { bw_min = std::min(bw_min, m.inter_Bpns); lat_max = std::max(lat_max, m.inter_lat_ns); }
    else
        for (uint32_t a = 0; a < N; a++)
            for (uint32_t b = 0; b < N; b++)
                if (a != b) { bw_min = std::min(bw_min, s->node_bw[a * N + b]); lat_max = std::max(lat_max, s->node_lat[a * N + b]); }
    std::vector<uint32_t> image = constants_image(m, s->intra_bw, s->intra_lat, s->node_bw, s->node_lat, s->ties);
    uint32_t* d_new = nullptr;
    int rc = upload(image, &d_new);
    if (rc) return rc;
    if (hipDeviceSynchronize() != hipSuccess) { hipFree(d_new); return FF_EHIP; }   // no launch may still read the old table
    hipFree(s->d_magic);
    s->d_magic = d_new;
    s->dev.link_table = s->intra_bw.empty() ? 0u : 1u;
    s->dev.node_table = s->node_bw.empty() ? 0u : 1u;
    s->dev.ties = s->ties.empty() ? 0u : 1u;
    s->links_gen++;
    s->wide = needs_wide(s->big_tensors, bw_min, lat_max, G);
    return FF_OK;
}

int ff_sim_set_links(ff_sim_t* s, const ff_linktable_t* links) {
    if (!s) return FF_EINVAL;
    const uint32_t G = s->mach.gpus_per_node;
    std::vector<uint32_t> bw, lat;
    if (links) {
        if (!links->Bpns || links->gpus_per_node != G) return FF_EINVAL;
        bw.assign(links->Bpns, links->Bpns + (size_t)G * G);
        lat.assign((size_t)G * G, 0);
        if (links->lat_ns) lat.assign(links->lat_ns, links->lat_ns + (size_t)G * G);
        for (uint32_t a = 0; a < G; a++)
            for (uint32_t b = 0; b < G; b++) {
                if (a == b) { bw[a * G + b] = std::max(bw[a * G + b], 1u); continue; }   // a device needs no link to itself
                if (bw[a * G + b] < 1) return FF_EINVAL;
            }
    }
    s->intra_bw.swap(bw);
    s->intra_lat.swap(lat);
    const int rc = apply_link_tables(s);
    if (rc) { s->intra_bw.swap(bw); s->intra_lat.swap(lat); }     // nothing changed on the device: keep the old table
    return rc;
}

int ff_sim_set_ties(ff_sim_t* s, const uint32_t* leader) {
    if (!s) return FF_EINVAL;
    std::vector<uint32_t> t;
    if (leader) {
        const uint32_t n = s->dev.n_ops;
        t.assign(leader, leader + n);
        for (uint32_t i = 0; i < n; i++)
            if (t[i] >= n || t[t[i]] != t[i]) return FF_EINVAL;      // a leader leads itself
    }
    s->ties.swap(t);
    const int rc = apply_link_tables(s);
    if (rc) s->ties.swap(t);
    return rc;
}

int ff_sim_set_node_links(ff_sim_t* s, const ff_nodelinks_t* links) {
    if (!s) return FF_EINVAL;
    const uint32_t N = s->mach.n_nodes;
    std::vector<uint32_t> bw, lat;
    if (links) {
        if (!links->Bpns || links->n_nodes != N) return FF_EINVAL;
        bw.assign(links->Bpns, links->Bpns + (size_t)N * N);
        lat.assign((size_t)N * N, 0);
        if (links->lat_ns) lat.assign(links->lat_ns, links->lat_ns + (size_t)N * N);
        for (uint32_t a = 0; a < N; a++)
            for (uint32_t b = 0; b < N; b++) {
                if (a == b) { bw[a * N + b] = std::max(bw[a * N + b], 1u); continue; }   // not used
                if (bw[a * N + b] < 1) return FF_EINVAL;
            }
    }
    s->node_bw.swap(bw);
    s->node_lat.swap(lat);
    const int rc = apply_link_tables(s);
    if (rc) { s->node_bw.swap(bw); s->node_lat.swap(lat); }
    return rc;
}

size_t ff_sim_workspace_bytes(const ff_sim_t* s, uint32_t B) {
    if (!s) return 0;
    if (s->lds_words) return 0;   // the whole per-candidate state lives in LDS
    return (size_t)std::max<uint32_t>(1, batch_slots(s, B)) * s->batch_slot_bytes;
}

int ff_sim_set_workspace(ff_sim_t* s, void* d_ws, size_t bytes) {
    if (!s || (!d_ws && bytes) || ((uintptr_t)d_ws & 255)) return FF_EINVAL;
    s->ws = d_ws;
    s->ws_bytes = bytes;
    return FF_OK;
}

int ff_sim_set_stats(ff_sim_t* s, ff_stats_t* d_stats) {
    if (!s) return FF_EINVAL;
    s->d_stats = d_stats;
    return FF_OK;
}

// Keeping the per-edge set-up costs LDS for graphs whose words live there; it is used unless it
// would leave part of the batch waiting for a free compute unit that the plain variant has room for.
static bool batch_cached(const ff_sim* s, uint32_t B) {
    return s->cache_ok && (B <= s->max_slots_cached || s->max_slots_cached >= s->max_slots);
}
// wavefronts (= workspace slots) a launch of B candidates uses
static uint32_t batch_slots(const ff_sim* s, uint32_t B) {
    return std::min(B, batch_cached(s, B) ? s->max_slots_cached : s->max_slots);
}

static int batch_impl(ff_sim_t* s, const ff_opcfg_t* d_strategies, const uint16_t* d_devmaps, uint32_t B, uint64_t* d_out_ns,
                      void* hip_stream) {
    if (!s || (B && (!d_strategies || !d_out_ns))) return FF_EINVAL;
    if (B == 0) return FF_OK;
    const int ext = ext_level(s, d_devmaps != nullptr);
    const bool cached = batch_cached(s, B);
    const uint32_t slots = batch_slots(s, B);
    if (!s->lds_words && (!s->ws || s->ws_bytes < (size_t)slots * s->batch_slot_bytes)) return FF_EWORKSPACE;
    hipStream_t st = (hipStream_t)hip_stream;
    static_assert(sizeof(Counters) == sizeof(ff_stats_t), "stats layout");
    if (!allow_lds((const void*)batch_kernel(s, cached, ext), cached ? s->lds_cached : s->lds)) return FF_EHIP;
    hipLaunchKernelGGL(batch_kernel(s, cached, ext), dim3(slots), dim3(WAVE), cached ? s->lds_cached : s->lds, st, s->dev, s->d_ops,
                       s->d_edges, s->d_in_edges, s->d_cost, s->d_magic, (const uint2*)d_strategies, B, (u64*)d_out_ns,
                       (Counters*)s->d_stats, (unsigned char*)s->ws, s->batch_slot_bytes, d_devmaps);
    return hipGetLastError() == hipSuccess ? FF_OK : FF_EHIP;
}

int ff_sim_batch_kernel_name(const ff_sim_t* s, uint32_t B, char* buf, size_t len) {
    if (!s || !buf || len < 1) return FF_EINVAL;
    const int ext = ext_level(s);
    const KernelChoice k = choice(s, batch_cached(s, B));
    const int n = snprintf(buf, len, "k_sim_batch<%s, %s, %s, %d, %s, %d, %d>", k.wide ? "true" : "false", k.lds_words ? "true" : "false",
                           k.stats ? "true" : "false", batch_queue_shape(k), k.cache ? "true" : "false", ext,
                           s->dev.gpus_per_node == 4 ? 4 : 0);
    return (n < 0 || (size_t)n >= len) ? FF_ERANGE : FF_OK;
}

int ff_sim_accept_table(double beta_per_ns, uint64_t bucket_ns, uint32_t n_buckets, uint32_t* out) {
    if (!out || n_buckets < 1 || bucket_ns < 1 || !(beta_per_ns >= 0.0)) return FF_EINVAL;
    for (uint32_t b = 0; b < n_buckets; b++) {
        // probability of accepting a proposal at the lower edge of bucket b, scaled by 2^32
        const double p = std::exp(-beta_per_ns * (double)b * (double)bucket_ns) * 4294967296.0;
        out[b] = p >= 4294967295.0 ? 0xffffffffu : (uint32_t)std::floor(p);
    }
    return FF_OK;
}

int ff_sim_batch(ff_sim_t* s, const ff_opcfg_t* d_strategies, uint32_t B, uint64_t* d_out_ns, void* hip_stream) {
    return batch_impl(s, d_strategies, nullptr, B, d_out_ns, hip_stream);
}

int ff_sim_batch_devmaps(ff_sim_t* s, const ff_opcfg_t* d_strategies, const uint16_t* d_devmaps, uint32_t B, uint64_t* d_out_ns,
                         void* hip_stream) {
    if (B && !d_devmaps) return FF_EINVAL;
    return batch_impl(s, d_strategies, d_devmaps, B, d_out_ns, hip_stream);
}

static int launch_chain_steps(ff_chains* c, const ff_mutation_t* d_muts, uint32_t n_steps, uint64_t* d_out, hipStream_t st,
                              const SearchDev& search) {
    ff_sim* s = c->sim;
    static_assert(sizeof(ff_mutation_t) == 12, "mutation layout");
    if (!allow_lds((const void*)chain_kernel(s), s->lds_chain)) return FF_EHIP;
    hipLaunchKernelGGL(chain_kernel(s), dim3(c->C), dim3(WAVE), s->lds_chain, st, s->dev, s->d_ops, s->d_edges, s->d_in_edges,
                       s->d_cost, s->d_magic, c->d_mem, c->stride, c->n_snaps, c->C, (const uint32_t*)d_muts, n_steps,
                       (u64*)d_out, c->d_flags, search);
    return hipGetLastError() == hipSuccess ? FF_OK : FF_EHIP;
}

int ff_sim_chains_create(ff_sim_t* s, const ff_opcfg_t* d_strategies, uint32_t C, uint64_t* d_out_ns0, void* hip_stream,
                         ff_chains_t** out) {
    if (!out) return FF_EINVAL;
    *out = nullptr;
    if (!s || !d_strategies || !d_out_ns0 || C < 1) return FF_EINVAL;
    ff_chains* c = new (std::nothrow) ff_chains;
    if (!c) return FF_ENOMEM;
    c->sim = s;
    c->C = C;
    c->n_snaps = CHAIN_SNAPSHOTS;
    c->stride = chain_bytes(s->dev.n_ops, s->dev.n_ops_pad, s->dev.n_rows, c->n_snaps, s->dev.n_edges);
    hipStream_t st = (hipStream_t)hip_stream;
    const size_t row_bytes = (size_t)s->dev.n_ops * sizeof(uint2);
    if (hipMalloc((void**)&c->d_mem, (size_t)C * c->stride) != hipSuccess ||
        hipMalloc((void**)&c->d_flags, (size_t)C * 4) != hipSuccess ||
        hipMalloc((void**)&c->d_counter, 256) != hipSuccess) { ff_sim_chains_destroy(c); return FF_ENOMEM; }
    // zero everything (snapshot bookkeeping starts empty), then drop each chain's strategy at
    // the head of its block
    if (hipMemsetAsync(c->d_mem, 0, (size_t)C * c->stride, st) != hipSuccess ||
        hipMemsetAsync(c->d_flags, 0, (size_t)C * 4, st) != hipSuccess ||
        hipMemcpy2DAsync(c->d_mem, c->stride, d_strategies, row_bytes, row_bytes, C, hipMemcpyDeviceToDevice, st) != hipSuccess) {
        ff_sim_chains_destroy(c);
        return FF_EHIP;
    }
    int rc = launch_chain_steps(c, nullptr, 1, d_out_ns0, st, SearchDev{});
    if (rc) { ff_sim_chains_destroy(c); return rc; }
    c->links_gen = s->links_gen;
    *out = c;
    return FF_OK;
}

int ff_sim_delta(ff_chains_t* c, const ff_mutation_t* d_muts, uint32_t n_steps, uint64_t* d_out_ns, void* hip_stream) {
    if (!c || (n_steps && (!d_muts || !d_out_ns))) return FF_EINVAL;
    if (c->links_gen != c->sim->links_gen) return FF_EINVAL;
    if (n_steps == 0) return FF_OK;
    return launch_chain_steps(c, d_muts, n_steps, d_out_ns, (hipStream_t)hip_stream, SearchDev{});
}

// checks the search parameters and fills what the kernels take of them
static int search_params(ff_chains_t* c, const ff_search_t* p, SearchDev* out) {
    if (c->links_gen != c->sim->links_gen) return FF_EINVAL;
    if (!p->d_accept || !p->d_tuple_ptr || !p->d_tuples || !p->d_best_ns || !p->d_best || p->n_buckets < 1 || p->bucket_ns < 1 ||
        p->n_tuples < 1) return FF_EINVAL;
    // the per-op ranges index the tuple list on the device: they are read back and checked when a
    // chain set sees a list for the first time; later calls with the same list only launch
    if (c->checked_ptr != p->d_tuple_ptr || c->checked_n != p->n_tuples) {
        const uint32_t n_ops = c->sim->dev.n_ops;
        std::vector<uint32_t> ptr(n_ops + 1);
        if (hipMemcpy(ptr.data(), p->d_tuple_ptr, ptr.size() * 4, hipMemcpyDeviceToHost) != hipSuccess) return FF_EHIP;
        for (uint32_t i = 0; i < n_ops; i++)
            if (ptr[i] > ptr[i + 1] || ptr[i + 1] > p->n_tuples) return FF_EINVAL;
        c->checked_ptr = p->d_tuple_ptr;
        c->checked_n = p->n_tuples;
    }
    SearchDev sd{};
    sd.seed = p->seed; sd.first_step = p->first_step; sd.bucket_ns = p->bucket_ns;
    sd.accept = p->d_accept; sd.tuple_ptr = p->d_tuple_ptr; sd.tuples = p->d_tuples;
    sd.n_buckets = p->n_buckets; sd.enabled = 1; sd.patience = p->patience; sd.n_tuples = p->n_tuples;
    sd.best_ns = (u64*)p->d_best_ns; sd.best_cfgs = (uint2*)p->d_best;
    *out = sd;
    return FF_OK;
}

int ff_sim_search(ff_chains_t* c, const ff_search_t* p, uint32_t n_steps, uint64_t* d_trace_ns, void* hip_stream) {
    if (!c || !p || (n_steps && !d_trace_ns)) return FF_EINVAL;
    if (n_steps == 0) return c->links_gen != c->sim->links_gen ? FF_EINVAL : FF_OK;
    SearchDev sd{};
    const int rc = search_params(c, p, &sd);
    if (rc) return rc;
    return launch_chain_steps(c, nullptr, n_steps, d_trace_ns, (hipStream_t)hip_stream, sd);
}

// the trial kernel on M proposals per chain (d_muts [M][C]); the caller has checked the workspace
static int launch_trials(ff_chains* c, const uint32_t* d_muts, uint32_t M, uint64_t* d_out_ns, hipStream_t st) {
    ff_sim* s = c->sim;
    const uint32_t total = M * c->C;
    const uint32_t slots = std::min(total, s->max_try_slots);
    hipLaunchKernelGGL(k_zero_u32, dim3(1), dim3(WAVE), 0, st, c->d_counter);
    if (!allow_lds((const void*)try_kernel(s), s->lds_common)) return FF_EHIP;
    hipLaunchKernelGGL(try_kernel(s), dim3(slots), dim3(WAVE), s->lds_common, st, s->dev, s->d_ops, s->d_edges,
                       s->d_in_edges, s->d_cost, s->d_magic, c->d_mem, c->stride, c->n_snaps, c->C, d_muts, M,
                       (u64*)d_out_ns, c->d_flags, c->d_counter, (unsigned char*)s->ws, s->slot_bytes);
    return hipGetLastError() == hipSuccess ? FF_OK : FF_EHIP;
}

int ff_sim_search_ahead(ff_chains_t* c, const ff_search_t* p, uint32_t n_steps, uint32_t max_ahead, uint64_t* d_trace_ns,
                        void* hip_stream, ff_ahead_stats_t* h_stats) {
    const bool always = (max_ahead & FF_AHEAD_ALWAYS) != 0;
    max_ahead &= ~FF_AHEAD_ALWAYS;
    if (!c || !p || (n_steps && !d_trace_ns) || max_ahead < 1) return FF_EINVAL;
    if (h_stats) *h_stats = ff_ahead_stats_t{0, 0, 0, 0};
    if (n_steps == 0) return c->links_gen != c->sim->links_gen ? FF_EINVAL : FF_OK;
    SearchDev sd{};
    int rc = search_params(c, p, &sd);
    if (rc) return rc;
    ff_sim* s = c->sim;
    hipStream_t st = (hipStream_t)hip_stream;
    // no more proposals in flight than the trial kernel has wavefronts for
    const uint64_t fit = std::max<uint64_t>(1, (uint64_t)s->max_try_slots / c->C);
    const uint32_t cap = (uint32_t)std::min<uint64_t>(std::min<uint64_t>(max_ahead, fit), n_steps);
    {
        const uint32_t slots = (uint32_t)std::min<uint64_t>((uint64_t)cap * c->C, s->max_try_slots);
        if (!s->ws || s->ws_bytes < (size_t)slots * s->slot_bytes) return FF_EWORKSPACE;
    }
    if (cap < 4 && !always) {
        // the chains alone fill the device (or the caller allows no look-ahead worth a round): ff_sim_search
        rc = launch_chain_steps(c, nullptr, n_steps, d_trace_ns, st, sd);
        if (rc) return rc;
        if (hipStreamSynchronize(st) != hipSuccess) return FF_EHIP;
        if (h_stats) *h_stats = ff_ahead_stats_t{1, (uint64_t)n_steps * c->C, (uint64_t)n_steps * c->C, 0};
        return FF_OK;
    }
    if (c->ahead_cap < cap) {
        hipFree(c->d_ahead_muts); hipFree(c->d_ahead_ns); hipFree(c->d_ahead_done);
        c->d_ahead_muts = nullptr; c->d_ahead_ns = nullptr; c->d_ahead_done = nullptr; c->ahead_cap = 0;
        if (hipMalloc((void**)&c->d_ahead_muts, (size_t)cap * c->C * 12) != hipSuccess ||
            hipMalloc((void**)&c->d_ahead_ns, (size_t)cap * c->C * 8) != hipSuccess ||
            hipMalloc((void**)&c->d_ahead_done, (size_t)c->C * 8) != hipSuccess) return FF_ENOMEM;   // positions, then counts
        c->ahead_cap = cap;
    }
    hipLaunchKernelGGL(k_zero_words, dim3((2 * c->C + 255) / 256), dim3(256), 0, st, c->d_ahead_done, 2 * c->C);
    sd.done = c->d_ahead_done;
    sd.n_accepted = c->d_ahead_done + c->C;
    std::vector<uint32_t> now(2 * (size_t)c->C, 0), before;
    // Simulating ahead pays when few proposals are taken: a round costs about two simulations (the proposals side
    // by side, then the one that is taken) and advances a chain to its first accepted proposal.  The share of
    // accepted proposals is measured as the search goes (it falls as the chains settle); while it is high, or when
    // the chains alone fill the device, the steps are simulated one by one as in ff_sim_search.
    // A stretch without look-ahead: the first of a row is 8 steps, timed; the following ones end by the device's
    // clock, each four times as long as the one before (no chain waits for a slower one: each stops where it is).
    int clock_khz = 0;
    int dev_id = 0;
    if (hipGetDevice(&dev_id) != hipSuccess || hipDeviceGetAttribute(&clock_khz, hipDeviceAttributeWallClockRate, dev_id) != hipSuccess)
        clock_khz = 0;
    double stretch_ms = 0.0;               // length of the last stretch of the current row (0: none yet)
    double taken_share = 1.0;
    for (;;) {
        uint32_t K = 0;
        if (always) K = cap;
        else if (taken_share < 0.25) K = (uint32_t)std::min<double>(cap, std::max(4.0, 2.0 / std::max(taken_share, 1e-3)));
        sd.ahead_ns = K ? (const u64*)c->d_ahead_ns : nullptr;
        sd.n_ahead = K ? K : 8;
        sd.time_limit = 0;
        if (!K && stretch_ms > 0.0 && clock_khz > 0) {
            sd.n_ahead = n_steps;
            sd.time_limit = (u64)(4.0 * stretch_ms * clock_khz);
        }
        const auto t_begin = std::chrono::steady_clock::now();
        if (K) {
            const uint32_t n = K * c->C;
            hipLaunchKernelGGL(k_search_ahead_proposals, dim3((n + 255) / 256), dim3(256), 0, st, sd, s->dev.n_ops, s->dev.n_dev, c->C,
                               n_steps, c->d_ahead_muts);
            if ((rc = launch_trials(c, c->d_ahead_muts, K, c->d_ahead_ns, st))) return rc;
        }
        if ((rc = launch_chain_steps(c, nullptr, n_steps, d_trace_ns, st, sd))) return rc;
        before = now;
        if (hipMemcpyAsync(now.data(), c->d_ahead_done, now.size() * 4, hipMemcpyDeviceToHost, st) != hipSuccess ||
            hipStreamSynchronize(st) != hipSuccess) return FF_EHIP;
        uint64_t advanced = 0, active = 0, unfinished = 0, taken = 0;
        for (uint32_t k = 0; k < c->C; k++) {
            if (before[k] < n_steps) { active++; advanced += now[k] - before[k]; taken += now[c->C + k] - before[c->C + k]; }
            if (now[k] < n_steps) unfinished++;
        }
        if (h_stats) { h_stats->rounds++; h_stats->proposals_simulated += K ? (uint64_t)K * active : advanced; h_stats->steps += advanced; h_stats->accepted += taken; }
        if (!unfinished) break;
        if (advanced) taken_share = 0.5 * taken_share + 0.5 * (double)taken / (double)advanced;
        stretch_ms = K ? 0.0 : std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now() - t_begin).count();
    }
    return FF_OK;
}

// host copy of the per-op tuple ranges, validated; first[o - op_begin] = index of op o's first neighbour
static int neighbour_ranges(const ff_chains_t* c, const uint32_t* d_tuple_ptr, uint32_t n_tuples, uint32_t op_begin, uint32_t op_end,
                            std::vector<uint32_t>* first, uint64_t* total) {
    const uint32_t n_ops = c->sim->dev.n_ops;
    if (op_begin > op_end || op_end > n_ops) return FF_EINVAL;
    std::vector<uint32_t> ptr(n_ops + 1);
    if (hipMemcpy(ptr.data(), d_tuple_ptr, ptr.size() * 4, hipMemcpyDeviceToHost) != hipSuccess) return FF_EHIP;
    for (uint32_t i = 0; i < n_ops; i++)
        if (ptr[i] > ptr[i + 1] || ptr[i + 1] > n_tuples) return FF_EINVAL;
    first->assign(op_end - op_begin + 1, 0);
    uint64_t acc = 0;
    for (uint32_t o = op_begin; o < op_end; o++) {
        (*first)[o - op_begin] = (uint32_t)acc;
        acc += (uint64_t)(ptr[o + 1] - ptr[o]) * c->sim->dev.n_dev;
        if (acc > 0xffffffffull) return FF_ERANGE;
    }
    (*first)[op_end - op_begin] = (uint32_t)acc;
    *total = acc;
    return FF_OK;
}

int ff_sim_neighbour_count(const ff_chains_t* c, const uint32_t* d_tuple_ptr, uint32_t n_tuples, uint32_t op_begin, uint32_t op_end,
                           uint32_t* out_count) {
    if (!c || !d_tuple_ptr || !out_count) return FF_EINVAL;
    std::vector<uint32_t> first;
    uint64_t total = 0;
    const int rc = neighbour_ranges(c, d_tuple_ptr, n_tuples, op_begin, op_end, &first, &total);
    if (rc) return rc;
    *out_count = (uint32_t)total;
    return FF_OK;
}

int ff_sim_neighbours(ff_chains_t* c, const uint32_t* d_tuple_ptr, const uint32_t* d_tuples, uint32_t n_tuples, uint32_t op_begin,
                      uint32_t op_end, ff_mutation_t* d_muts, uint64_t* d_out_ns, uint64_t* d_best_ns, uint32_t* d_best_index,
                      void* hip_stream) {
    if (!c || !d_tuple_ptr || !d_tuples || !d_muts || !d_out_ns || !d_best_ns || !d_best_index) return FF_EINVAL;
    if (c->links_gen != c->sim->links_gen) return FF_EINVAL;
    std::vector<uint32_t> first;
    uint64_t total = 0;
    int rc = neighbour_ranges(c, d_tuple_ptr, n_tuples, op_begin, op_end, &first, &total);
    if (rc) return rc;
    if (total == 0) return FF_EINVAL;
    if (total * c->C > 0xffffffffull) return FF_ERANGE;
    const uint32_t M = (uint32_t)total;
    hipStream_t st = (hipStream_t)hip_stream;
    // the index ranges of the ops: a small allocation of the library's for the duration of the call
    uint32_t* d_first = nullptr;
    if (hipMalloc(&d_first, first.size() * 4) != hipSuccess) return FF_ENOMEM;
    if (hipMemcpyAsync(d_first, first.data(), first.size() * 4, hipMemcpyHostToDevice, st) != hipSuccess ||
        hipStreamSynchronize(st) != hipSuccess) { hipFree(d_first); return FF_EHIP; }   // `first` is pageable host memory
    hipLaunchKernelGGL(k_neighbour_list, dim3((M + WAVE - 1) / WAVE), dim3(WAVE), 0, st, d_tuple_ptr, d_tuples, d_first, op_begin,
                       op_end, c->sim->dev.n_dev, M, c->C, (uint32_t*)d_muts, (const uint32_t*)nullptr);
    rc = ff_sim_delta_try(c, d_muts, M, d_out_ns, hip_stream);
    if (rc == FF_OK) {
        hipLaunchKernelGGL(k_best_of, dim3(c->C), dim3(WAVE), 0, st, (const u64*)d_out_ns, M, c->C, (u64*)d_best_ns, d_best_index);
        if (hipGetLastError() != hipSuccess) rc = FF_EHIP;
    }
    // the list kernel is the only reader of d_first
    if (hipStreamSynchronize(st) != hipSuccess && rc == FF_OK) rc = FF_EHIP;
    hipFree(d_first);
    return rc;
}

int ff_sim_neighbours_noalloc(ff_chains_t* c, const uint32_t* d_tuple_ptr, const uint32_t* d_tuples, uint32_t n_tuples, uint32_t op_begin,
                              uint32_t op_end, uint32_t M, ff_mutation_t* d_muts, uint64_t* d_out_ns, uint64_t* d_best_ns,
                              uint32_t* d_best_index, void* hip_stream) {
    if (!c || !d_tuple_ptr || !d_tuples || !d_muts || !d_out_ns || !d_best_ns || !d_best_index) return FF_EINVAL;
    if (c->links_gen != c->sim->links_gen) return FF_EINVAL;
    if (op_begin >= op_end || op_end > c->sim->dev.n_ops || M == 0) return FF_EINVAL;
    if (op_end - op_begin > NEIGHBOUR_SCRATCH_OPS) return FF_ERANGE;
    if ((uint64_t)M * c->C > 0xffffffffull) return FF_ERANGE;
    uint32_t* scratch = neighbour_scratch_of_current_device();
    if (!scratch) return FF_EHIP;
    hipStream_t st = (hipStream_t)hip_stream;
    uint32_t* d_first = scratch;
    uint32_t* d_status = scratch + NEIGHBOUR_SCRATCH_OPS + 1;
    hipLaunchKernelGGL(k_neighbour_first, dim3(1), dim3(WAVE), 0, st, d_tuple_ptr, n_tuples, op_begin, op_end, c->sim->dev.n_dev, M,
                       d_first, d_status);
    hipLaunchKernelGGL(k_neighbour_list, dim3((M + WAVE - 1) / WAVE), dim3(WAVE), 0, st, d_tuple_ptr, d_tuples, (const uint32_t*)d_first,
                       op_begin, op_end, c->sim->dev.n_dev, M, c->C, (uint32_t*)d_muts, (const uint32_t*)d_status);
    if (hipGetLastError() != hipSuccess) return FF_EHIP;
    int rc = ff_sim_delta_try(c, d_muts, M, d_out_ns, hip_stream);
    if (rc != FF_OK) return rc;
    hipLaunchKernelGGL(k_best_of, dim3(c->C), dim3(WAVE), 0, st, (const u64*)d_out_ns, M, c->C, (u64*)d_best_ns, d_best_index);
    return hipGetLastError() == hipSuccess ? FF_OK : FF_EHIP;
}

size_t ff_sim_delta_try_workspace_bytes(const ff_chains_t* c, uint32_t M) {
    if (!c) return 0;
    const uint64_t total = (uint64_t)M * c->C;
    return (size_t)std::max<uint64_t>(1, std::min<uint64_t>(total, c->sim->max_try_slots)) * c->sim->slot_bytes;
}

int ff_sim_delta_try(ff_chains_t* c, const ff_mutation_t* d_muts, uint32_t M, uint64_t* d_out_ns, void* hip_stream) {
    if (!c || (M && (!d_muts || !d_out_ns))) return FF_EINVAL;
    if (c->links_gen != c->sim->links_gen) return FF_EINVAL;
    if (M == 0) return FF_OK;
    if ((uint64_t)M * c->C > 0xffffffffull) return FF_ERANGE;
    ff_sim* s = c->sim;
    const uint32_t total = M * c->C;
    const uint32_t slots = std::min(total, s->max_try_slots);
    if (!s->ws || s->ws_bytes < (size_t)slots * s->slot_bytes) return FF_EWORKSPACE;
    return launch_trials(c, (const uint32_t*)d_muts, M, d_out_ns, (hipStream_t)hip_stream);
}

int ff_sim_chains_get_stats(ff_chains_t* c, ff_chain_stats_t* h_out) {
    if (!c || !h_out) return FF_EINVAL;
    if (hipDeviceSynchronize() != hipSuccess) return FF_EHIP;
    for (uint32_t k = 0; k < c->C; k++) {
        ChainMeta meta;
        const unsigned char* p = c->d_mem + (size_t)k * c->stride + chain_meta_offset(c->sim->dev.n_ops, c->sim->dev.n_ops_pad, c->sim->dev.n_rows, c->n_snaps, c->sim->dev.n_edges);
        if (hipMemcpy(&meta, p, sizeof(meta), hipMemcpyDeviceToHost) != hipSuccess) return FF_EHIP;
        h_out[k].n_steps = meta.n_steps;
        h_out[k].n_resumed = meta.n_resumed;
        h_out[k].n_events = meta.n_events;
        h_out[k].n_events_full = meta.n_events_full;
        h_out[k].n_converged = meta.n_converged;
    }
    return FF_OK;
}

void ff_sim_chains_destroy(ff_chains_t* c) {
    if (!c) return;
    hipFree(c->d_mem);
    hipFree(c->d_flags);
    hipFree(c->d_counter);
    hipFree(c->d_ahead_muts);
    hipFree(c->d_ahead_ns);
    hipFree(c->d_ahead_done);
    delete c;
}

}  // extern "C"
