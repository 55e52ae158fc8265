// Configurations, the geometry of parts (boxes, devices, the range of an input a part reads), the
// context of one candidate, the kept per-edge set-up and the validity check (Section 4, and the
// pair enumeration of Section 5.1 step 2 in closed form).
#pragma once
#include "ffsim_device.h"

namespace ffsim {

// up to this many groups of 64 ops the queue has no level 2: lanes scan level 1 directly
constexpr uint32_t FLAT_GROUPS = 8;
// GPUs per node up to which transfers are serialised on their link rows by a running sum
// along consecutive lanes (one shift per GPU); beyond, the general search for equal rows runs
constexpr uint32_t MAX_RUN = 8;

// Section timing for diagnostic builds (-DFFSIM_PROFILE): shader-clock ticks per section of the
// event loop are accumulated in registers and reported through the optional per-candidate record
// INSTEAD of its usual counters (section k in field k: 0 set-up, 1 queue pop, 2 wait for the popped
// op's words, 3 dequeue of READY tasks, 4 release: before the loop over producer parts, 5 wait
// for the edge's loads, 6 loop over producer parts, 7 consumer words and queue update).  Every mark
// reads the clock through the scalar memory path and waits for it, so LDS and scalar loads in
// flight are charged to the section that issued them; sections 2 and 5 wait for the vector loads.
// Compiled out otherwise.
#ifdef FFSIM_PROFILE
#define PROF_DECL u64 prof_t[8] = {cnt.exit_code, 0, 0, 0, 0, 0, 0, 0}; u64 prof_last = __builtin_readcyclecounter();
#define PROF_MARK(k) { const u64 prof_now = __builtin_readcyclecounter(); prof_t[k] += prof_now - prof_last; prof_last = prof_now; }
#define PROF_VMWAIT(k) { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); PROF_MARK(k) }
#define PROF_STORE(c) { c.n_compute = prof_t[0]; c.n_pairs = prof_t[1]; c.n_comm = prof_t[2]; c.sum_comm_ns = lane_id() == 0 ? prof_t[3] : 0; \
                        c.n_events = prof_t[4]; c.exit_code = prof_t[5]; c.n_stuck = prof_t[6]; c.want_check = prof_t[7]; }
#else
#define PROF_DECL
#define PROF_MARK(k)
#define PROF_VMWAIT(k)
#define PROF_STORE(c)
#endif

struct Counters { u64 n_compute, n_pairs, n_comm, sum_comm_ns, n_events, exit_code, n_stuck, want_check; };

// read-only tables shared by all candidates (pointers come from __restrict__ kernel
// arguments, so loads through them can use the scalar unit)
struct Tables {
    const DOp* ops;
    const DEdge* edges;       // sorted by (producer, consumer)
    const DEdge* in_edges;    // the same records sorted by (consumer, edge id)
    const uint32_t* cost;     // [n_ops][n_cols]
};

// LDS of one wavefront
struct WaveLds {
    u64* free_at;     // [n_rows]    endTime of the last task on every device / link row
    u64* l1;          // [n_ops_pad] min word per op
    u64* l2;          // [64]        min word per group of 64 ops
    uint8_t* tag;     // [n_rows]    scratch for conflict detection between lanes
};

__host__ __device__ inline size_t lds_common_bytes(uint32_t n_rows, uint32_t n_ops_pad) {
    return (size_t)n_rows * 8 + (size_t)n_ops_pad * 8 + 64 * 8 + ((n_rows + 15) & ~15u);
}
// per-candidate task words + per-op exeTime: in LDS for small graphs, else in an HBM slot
// (five words per lane and edge, then, behind those of all edges, one more per lane and edge: the
// consumer's parts in (node, part) order, see EdgeLane::sortw)
__host__ __device__ inline size_t ecache_bytes(uint32_t n_edges) { return (size_t)n_edges * 6 * WAVE * 4; }
__host__ __device__ inline size_t slot_bytes(uint32_t n_ops, uint32_t n_ops_pad) {
    return (size_t)n_ops * WAVE * 8 + (size_t)n_ops_pad * 4;
}

__device__ __forceinline__ WaveLds carve_lds(unsigned char* base, const SimDev& S) {
    WaveLds L;
    L.free_at = (u64*)base;
    L.l1 = L.free_at + S.n_rows;
    L.l2 = L.l1 + S.n_ops_pad;
    L.tag = (uint8_t*)(L.l2 + 64);
    return L;
}

struct OpCfg { uint32_t deg[4]; uint32_t off, stride, parts, x; };   // x = the four degrees, one byte each

// a configuration is the same for all lanes: keep it on the scalar unit
__device__ __forceinline__ OpCfg unpack_cfg(uint2 c) {
    OpCfg o;
    c.x = first_u32(c.x);
    c.y = first_u32(c.y);
    o.deg[0] = c.x & 0xff; o.deg[1] = (c.x >> 8) & 0xff; o.deg[2] = (c.x >> 16) & 0xff; o.deg[3] = c.x >> 24;
    o.off = c.y & 0xffff; o.stride = c.y >> 16; o.x = c.x;
    o.parts = o.deg[0] * o.deg[1] * o.deg[2] * o.deg[3];
    return o;
}

// per-lane variant (each lane looks at a different op)
__device__ __forceinline__ OpCfg unpack_cfg_lane(uint2 c) {
    OpCfg o;
    o.deg[0] = c.x & 0xff; o.deg[1] = (c.x >> 8) & 0xff; o.deg[2] = (c.x >> 16) & 0xff; o.deg[3] = c.x >> 24;
    o.off = c.y & 0xffff; o.stride = c.y >> 16; o.x = c.x;
    o.parts = o.deg[0] * o.deg[1] * o.deg[2] * o.deg[3];
    return o;
}

// Section 4: validity of a configuration for its op
__device__ __forceinline__ bool cfg_ok(const DOp& op, const OpCfg& c, const SimDev& S) {
    bool ok = true;
#pragma unroll
    for (int d = 0; d < 4; d++) {
        bool par = (uint32_t)d < op.ndim && ((op.par_mask >> d) & 1);
        ok = ok && c.deg[d] >= 1 && (par ? c.deg[d] <= op.extent[d] : c.deg[d] == 1);
    }
    // each degree <= 255, so the product cannot wrap
    return ok && c.parts <= S.max_parts && c.off < S.n_dev;
}

// floor(n / d), d uniform in 1..64, n <= 2^26, without branches.  Lane d-1 of magic_v holds
// floor(2^32/d)+1 for d >= 2 and 0 for d = 1 (where the quotient is n itself), so the
// constant comes from a register instead of memory.
struct Divisor { uint32_t d, m, pass; };   // pass = all ones iff d == 1
__device__ __forceinline__ Divisor divisor(uint32_t d, uint32_t magic_v) {
    Divisor v;
    v.d = d;
    v.m = readlane_u32(magic_v, (int)((d - 1) & 63));
    v.pass = d == 1 ? 0xffffffffu : 0u;
    return v;
}
__device__ __forceinline__ uint32_t div_by(uint32_t n, const Divisor& v) { return __umulhi(n, v.m) + (n & v.pass); }
// lane l gets the multiply-high constant of the divisor l+1
__device__ __forceinline__ uint32_t load_magic(const uint32_t* __restrict__ magic) { return magic[lane_id() + 1]; }

// output box of part k of an op: [lo[d], hi[d]) (equal-size partitions, Section 4)
struct Box { uint32_t lo[4], hi[4]; };

__device__ __forceinline__ Box part_box(const uint32_t extent[4], const OpCfg& c, uint32_t k, uint32_t magic_v) {
    Box b;
    uint32_t rem = k;
#pragma unroll
    for (int d = 3; d >= 0; d--) {
        if (c.deg[d] == 1) {          // uniform: most dims are not split
            b.lo[d] = 0;
            b.hi[d] = extent[d];
        } else {
            const Divisor dv = divisor(c.deg[d], magic_v);
            uint32_t q = div_by(rem, dv);
            uint32_t idx = rem - q * c.deg[d];
            rem = q;
            b.lo[d] = div_by(idx * extent[d], dv);
            b.hi[d] = div_by((idx + 1) * extent[d], dv);
        }
    }
    return b;
}

// REG: stride 1 and k < parts <= n_dev, so off + k wraps around at most once
template <bool REG = false>
__device__ __forceinline__ uint32_t part_device(const OpCfg& c, uint32_t k, const SimDev& S) {
    if (REG) {
        const uint32_t n = c.off + (k < S.n_dev ? k : 0u);   // lanes beyond the parts stay in range
        return n >= S.n_dev ? n - S.n_dev : n;
    }
    uint32_t n = c.off + k * c.stride;
    return n - div_magic(n, S.magic_dev, S.pass_dev) * S.n_dev;
}

// index of part k along each dim (mixed radix over the degree tuple, dim 0 slowest), packed
// one byte per dim
__device__ __forceinline__ uint32_t part_digits(const OpCfg& c, uint32_t k, uint32_t magic_v) {
    uint32_t rem = k, packed = 0;
#pragma unroll
    for (int d = 3; d >= 0; d--) {
        if (c.deg[d] != 1) {          // uniform
            const Divisor dv = divisor(c.deg[d], magic_v);
            const uint32_t q = div_by(rem, dv);
            packed |= (rem - q * c.deg[d]) << (8 * d);
            rem = q;
        }
    }
    return packed;
}

// Range of the producer's dim read by a consumer part (Section 4: the input sub-tensor
// follows from the output sub-tensor).  m: the map of that producer dim; extent: the
// producer's extent; cfg_x: the consumer's four degrees (one byte each); digits: the consumer
// part's index per dim (part_digits).  All values fit 32 bits: extents <= 2^20, stride <= 1024,
// |a|,|b| <= 2^29.  No branch on the lane's data.
__device__ __forceinline__ void needed_range(const DMap& m, uint32_t extent, uint32_t cfg_x, uint32_t digits,
                                             uint32_t magic_v, int32_t& lo, int32_t& hi) {
    if (m.src_dim < 0) { lo = 0; hi = (int32_t)extent; return; }   // uniform
    const uint32_t sh = 8u * (uint32_t)m.src_dim;
    const uint32_t deg = (cfg_x >> sh) & 0xff;
    const int32_t E = (int32_t)extent;
    if (deg == 1) {
        // the consumer does not split this dim: every part reads the same range (scalar unit)
        int32_t l = m.a, h = ((int32_t)m.cext - 1) * (int32_t)m.stride + m.b + 1;
        l = l < 0 ? 0 : (l > E ? E : l);
        h = h < 0 ? 0 : (h > E ? E : h);
        lo = l;
        hi = h < l ? l : h;
        return;
    }
    const Divisor dv = divisor(deg, magic_v);
    const uint32_t idx = (digits >> sh) & 0xff;
    const int32_t clo = (int32_t)div_by(idx * m.cext, dv);
    const int32_t chi = (int32_t)div_by((idx + 1) * m.cext, dv);
    int32_t l = clo * (int32_t)m.stride + m.a;
    int32_t h = (chi - 1) * (int32_t)m.stride + m.b + 1;
    l = l < 0 ? 0 : (l > E ? E : l);
    h = h < 0 ? 0 : (h > E ? E : h);
    lo = l;
    hi = h < l ? l : h;
}

// index of the producer part (along one dim) that owns coordinate x: the largest p with
// floor(p*E/deg) <= x
__device__ __forceinline__ uint32_t owner_part(uint32_t x, uint32_t E, uint32_t deg) {
    return ((x + 1) * deg - 1) / E;
}

// Everything one wavefront needs to simulate its candidate.  cfgs is deliberately not
// __restrict__: the chain kernel rewrites a configuration between simulations, so loads
// from it must not be treated as invariant.
// OVR: one op's configuration may be overridden (trial mutations); the plain form does not
// pay for the comparison.
// EXT: 0, 1 or 2.  From 1 on: the refinements of the inputs that only some callers use -- links inside a node that
// differ per pair, explicit devices per task -- are compiled into kernels of their own; the
// plain kernels carry none of it.
// GPN: the machine's number of GPUs per node when the kernel is compiled for one (4: node and
// local index of a device are a shift and a mask, and three scalars fewer stay alive in the
// event loop), 0 = any.
template <bool OVR, int EXT = 0, int GPN = 0>
struct SimT {
    const SimDev& S;
    const Tables& T;
    const uint2* cfgs;       // the candidate's n_ops configurations
    u64* words;              // [n_ops*64] task words (LDS or HBM)
    uint32_t* exe_of;        // [n_ops] exeTime of the op's tasks under its configuration
    const WaveLds& L;
    uint32_t magic_v;
    u64 last_key;            // lower bound of every pending event word
    bool overflow;
    // a trial mutation: op ov_op is simulated with configuration ov_cfg instead of cfgs[ov_op]
    uint32_t ov_op;          // 0xffffffff = none
    uint2 ov_cfg;
    uint32_t* ecache;        // per (edge, consumer part) values kept from the set-up (see EdgeLane), or null
    bool ecache_fill;        // init_state writes them (false: ecache is someone else's and only read)
    const uint4* links = nullptr;        // per ordered pair of local GPUs: bandwidth, its magic, latency (S.link_table)
    const uint4* node_links = nullptr;   // per ordered pair of nodes: the same three figures (S.node_table)
    const uint16_t* devmap = nullptr;    // [n_ops][64] device of every part given explicitly, or null
    const uint32_t* tie = nullptr;       // [n_ops] tied configurations (S.ties), or null
    bool want_sort = false;              // the set-up of an edge includes the consumer's parts in (node, part) order (general event loop)
    static constexpr bool kOvr = OVR;
    static constexpr bool kExt = EXT >= 1;      // refinements of the inputs: link tables, explicit devices, parameter traffic
    static constexpr bool kTrain = EXT >= 2;    // training-iteration graphs: contributing edges, tied configurations
    static_assert(GPN == 0 || GPN == 4, "compiled node sizes");
    __device__ __forceinline__ uint32_t gpn() const { return GPN ? (uint32_t)GPN : S.gpus_per_node; }
    __device__ __forceinline__ uint32_t node_of(uint32_t dev) const {
        return GPN == 4 ? dev >> 2 : div_magic(dev, S.magic_gpn, S.pass_gpn);
    }
    __device__ __forceinline__ uint32_t local_of(uint32_t dev, uint32_t node) const {
        return GPN == 4 ? (dev & 3u) : dev - node * S.gpus_per_node;
    }
    // the op whose configuration op j takes (Section 4: one configuration per operation; the forward and the
    // backward computation of an operation are two ops of the graph)
    __device__ __forceinline__ uint32_t leader_of(uint32_t j) const { return (kTrain && tie) ? tie[j] : j; }
    __device__ __forceinline__ bool overridden(uint32_t j) const { return OVR && leader_of(j) == ov_op; }
    __device__ __forceinline__ uint2 cfg_raw(uint32_t j) const {
        j = leader_of(j);
        uint2 c = cfgs[j];
        if (OVR && j == ov_op) c = ov_cfg;
        return c;
    }
    __device__ __forceinline__ OpCfg cfg(uint32_t j) const { return unpack_cfg(cfg_raw(j)); }
    // Section 4: the device of this lane's part of op j (lanes beyond the parts get some device in range)
    template <bool REG>
    __device__ __forceinline__ uint32_t device_of(uint32_t j, const OpCfg& c) const { return device_of_part<REG>(j, c, lane_id()); }
    // the same for part k of op j (k may differ per lane)
    template <bool REG>
    __device__ __forceinline__ uint32_t device_of_part(uint32_t j, const OpCfg& c, uint32_t k) const {
        if (EXT && !REG && devmap) {
            // (the entry is requested before the number of parts is known; one beyond the parts is dropped)
            const uint32_t d = devmap[(size_t)j * WAVE + (k & (WAVE - 1))];
            return k < c.parts ? d : 0u;
        }
        return part_device<REG>(c, k, S);
    }
};
constexpr uint32_t NO_OVERRIDE = 0xffffffffu;
typedef SimT<false> Sim;
typedef SimT<true> SimTrial;

// What the release of an edge needs to know about each consumer part (one per lane).  It
// depends only on the edge and on the consumer's configuration, not on which producer part
// finished or when, and an edge is visited once per group of producer parts that finish
// together: the batch kernels compute it once per candidate and keep it (ECACHE_WORDS words per
// lane and edge, in LDS or in the candidate's HBM slot) when all extents fit 16 bits.
struct EdgeLane {
    int32_t nlo[4], nhi[4];     // range of every producer dim the part reads ([0,1) beyond the producer's dims)
    uint32_t dev_c, node_c;     // the part's device and node
    bool mine;                  // the lane is a part of the consumer
    // regular strategies: position inside the run of lanes that share a remote link row (see run_events)
    uint32_t pos, last_run_mask, first_len;
    bool run_end, wrapped;
    // general strategies: the consumer's parts in (node, part) order, so that the transfers from one producer part
    // that share a link row between two nodes are neighbours.  Bits 0-5: the part that sorts to this
    // lane's position; 6-11: this lane's part's position; 12-21: the node of the part at this position; 22: the
    // position starts a node (or lies beyond the parts); 23: this lane's part shares its device with a
    // lower part of the consumer.
    uint32_t sortw;
};
constexpr uint32_t ECACHE_WORDS = 5;
constexpr uint32_t ECACHE_MAX_EXTENT = 0xffff;

template <class SimX>
__device__ __forceinline__ EdgeLane edge_lane(const SimX& m, const DEdge& e, const OpCfg& cj) {
    const int lane = lane_id();
    const SimDev& S = m.S;
    EdgeLane el;
    el.mine = (uint32_t)lane < cj.parts;
    const uint32_t digits = part_digits(cj, lane, m.magic_v);
    if (SimX::kTrain && e.kind) {
        // a contributing edge: the ranges are taken in the consumer's own tensor, of which this lane's part holds a box
        const Box cb = part_box(e.src_extent, cj, lane, m.magic_v);
#pragma unroll
        for (int d = 0; d < 4; d++) {
            el.nlo[d] = (uint32_t)d < e.src_ndim ? (int32_t)cb.lo[d] : 0;
            el.nhi[d] = (uint32_t)d < e.src_ndim ? (int32_t)cb.hi[d] : 1;
        }
    } else {
#pragma unroll
        for (int d = 0; d < 4; d++) {
            el.nlo[d] = 0; el.nhi[d] = 1;
            if ((uint32_t)d < e.src_ndim) needed_range(e.map[d], e.src_extent[d], cj.x, digits, m.magic_v, el.nlo[d], el.nhi[d]);
        }
    }
    const uint32_t G = m.gpn();
    // the run fields only depend on the consumer's own configuration: filled whenever it puts its
    // parts on consecutive, distinct devices, whatever the other ops do
    const bool consecutive = cj.stride == 1 && cj.parts <= S.n_dev && G <= MAX_RUN && !(SimX::kExt && m.devmap);
    el.dev_c = consecutive ? part_device<true>(cj, lane, S) : m.template device_of<false>(e.dst, cj);
    el.node_c = m.node_of(el.dev_c);
    el.pos = 0; el.first_len = 0; el.last_run_mask = 0; el.run_end = false; el.wrapped = false;
    el.sortw = 0;
    if (m.want_sort) {
        uint32_t rank = 0;
        bool dup = false;
        for (uint32_t l2 = 0; l2 < cj.parts; l2++) {
            const uint32_t n2 = readlane_u32(el.node_c, (int)l2), d2 = readlane_u32(el.dev_c, (int)l2);
            rank += (n2 < el.node_c || (n2 == el.node_c && l2 < (uint32_t)lane)) ? 1u : 0u;
            dup = dup || (d2 == el.dev_c && l2 < (uint32_t)lane);
        }
        const uint32_t spos = el.mine ? rank : (uint32_t)lane;       // lanes beyond the parts stay where they are
        const uint32_t part_here = scatter_u32((uint32_t)lane, spos);
        const uint32_t node_here = scatter_u32(el.node_c, spos);
        const uint32_t node_before = wave_shr1_u32(node_here);
        const bool head = lane == 0 || (uint32_t)lane >= cj.parts || node_here != node_before;
        el.sortw = part_here | (spos << 6) | (node_here << 12) | ((uint32_t)head << 22) | ((uint32_t)(dup && el.mine) << 23);
    }
    if (consecutive) {
        const uint32_t node0 = m.node_of(cj.off);
        const uint32_t room = G - (cj.off - node0 * G);              // lanes of the first run
        el.first_len = cj.parts < room ? cj.parts : room;
        const uint32_t local_c = m.local_of(el.dev_c, el.node_c);
        el.pos = (uint32_t)lane < el.first_len ? (uint32_t)lane : local_c;    // index inside the run
        const uint32_t last = cj.off + cj.parts - 1;
        el.wrapped = last >= S.n_dev && m.node_of(last - S.n_dev) == node0;
        el.last_run_mask = (el.wrapped && (uint32_t)lane >= el.first_len && el.node_c == node0) ? 0xffffffffu : 0u;
        el.run_end = el.mine && ((uint32_t)lane == cj.parts - 1 || local_c == G - 1) &&
                     !(el.wrapped && (uint32_t)lane == el.first_len - 1);
    }
    return el;
}

// ranges as lo | hi << 16; one word of small fields: device 10 bits, node 10, pos 3, run_end,
// last run, mine, first_len 4, wrapped
__device__ __forceinline__ void ecache_store(uint32_t* ecache, uint32_t n_edges, uint32_t eid, const EdgeLane& el) {
    ecache[(size_t)n_edges * (ECACHE_WORDS * WAVE) + (size_t)eid * WAVE + lane_id()] = el.sortw;
    uint32_t* p = ecache + (size_t)eid * (ECACHE_WORDS * WAVE) + lane_id();
#pragma unroll
    for (int d = 0; d < 4; d++) p[d * WAVE] = (uint32_t)el.nlo[d] | ((uint32_t)el.nhi[d] << 16);
    p[4 * WAVE] = el.dev_c | (el.node_c << 10) | (el.pos << 20) | ((uint32_t)el.run_end << 23) | ((el.last_run_mask & 1u) << 24) |
                  ((uint32_t)el.mine << 25) | (el.first_len << 26) | ((uint32_t)el.wrapped << 30);
}
__device__ __forceinline__ EdgeLane ecache_load(const uint32_t* ecache, uint32_t eid) {
    const uint32_t* p = ecache + (size_t)eid * (ECACHE_WORDS * WAVE) + lane_id();
    uint32_t v[ECACHE_WORDS];
#pragma unroll
    for (int k = 0; k < (int)ECACHE_WORDS; k++) v[k] = p[k * WAVE];
    EdgeLane el;
#pragma unroll
    for (int d = 0; d < 4; d++) { el.nlo[d] = (int32_t)(v[d] & 0xffffu); el.nhi[d] = (int32_t)(v[d] >> 16); }
    const uint32_t f = v[4];
    el.dev_c = f & 1023u; el.node_c = (f >> 10) & 1023u; el.pos = (f >> 20) & 7u;
    el.run_end = (f >> 23) & 1u; el.last_run_mask = 0u - ((f >> 24) & 1u); el.mine = (f >> 25) & 1u;
    const uint32_t u = first_u32(f);                 // the last two fields are the same in every lane
    el.first_len = (u >> 26) & 15u; el.wrapped = (u >> 30) & 1u;
    el.sortw = 0;
    return el;
}
__device__ __forceinline__ uint32_t ecache_sort_word(const uint32_t* ecache, uint32_t n_edges, uint32_t eid) {
    return ecache[(size_t)n_edges * (ECACHE_WORDS * WAVE) + (size_t)eid * WAVE + lane_id()];
}

// The number of inputs a consumer part has through a contributing edge: how many producer parts contribute to the box [blo, bhi) of the
// consumer's tensor.  Every dim of that tensor follows one producer dim (or none), so the count is a product
// over the PRODUCER's dims of the number of indices along that dim whose range meets the box in every dim that
// follows it (all indices, if none does).  Loops over the producer's degrees; runs once per edge and candidate.
__device__ __forceinline__ uint32_t count_contributors(const DEdge& e, const OpCfg& cp, const int32_t blo[4], const int32_t bhi[4], uint32_t magic_v) {
    uint32_t n = 1;
    for (int c = 0; c < 4; c++) {
        const uint32_t deg = cp.deg[c];
        uint32_t followers = 0;
        for (int d = 0; d < 4; d++) followers |= ((uint32_t)d < e.src_ndim && e.map[d].src_dim == c) ? (1u << d) : 0u;
        if (!followers) { n *= deg; continue; }
        const Divisor dv = divisor(deg, magic_v);
        uint32_t cnt = 0;
        for (uint32_t idx = 0; idx < deg; idx++) {
            bool meets = true;
            for (int d = 0; d < 4; d++) {
                if (!((followers >> d) & 1u)) continue;
                const DMap mp = e.map[d];
                const int32_t E = (int32_t)e.src_extent[d];
                const int32_t plo = (int32_t)div_by(idx * mp.cext, dv), phi = (int32_t)div_by((idx + 1) * mp.cext, dv);
                int32_t l = plo * (int32_t)mp.stride + mp.a, h = (phi - 1) * (int32_t)mp.stride + mp.b + 1;
                l = l < 0 ? 0 : (l > E ? E : l);
                h = h < 0 ? 0 : (h > E ? E : h);
                meets = meets && h > l && h > blo[d] && l < bhi[d];
            }
            cnt += meets ? 1u : 0u;
        }
        n *= cnt;
    }
    return n;
}

// how many parts of the producer (configuration cp) a consumer part reads through edge e:
// the product over the producer's dims of the number of producer parts its range touches
template <bool TRAIN = false>
__device__ __forceinline__ uint32_t count_inputs(const DEdge& e, const OpCfg& cp, uint32_t cons_cfg_x, uint32_t digits, uint32_t magic_v) {
    if (TRAIN && e.kind) {
        // this lane's box of the consumer's tensor
        int32_t blo[4], bhi[4];
#pragma unroll
        for (int d = 0; d < 4; d++) {
            const uint32_t deg = (cons_cfg_x >> (8 * d)) & 0xff, idx = (digits >> (8 * d)) & 0xff;
            blo[d] = 0; bhi[d] = (uint32_t)d < e.src_ndim ? (int32_t)e.src_extent[d] : 1;
            if (deg != 1) {
                const Divisor dv = divisor(deg, magic_v);
                blo[d] = (int32_t)div_by(idx * e.src_extent[d], dv);
                bhi[d] = (int32_t)div_by((idx + 1) * e.src_extent[d], dv);
            }
        }
        return count_contributors(e, cp, blo, bhi, magic_v);
    }
    uint32_t n = 1;
#pragma unroll
    for (int d = 0; d < 4; d++) {
        if ((uint32_t)d < e.src_ndim) {
            if (e.map[d].src_dim < 0) {
                n *= cp.deg[d];
            } else {
                int32_t lo, hi;
                needed_range(e.map[d], e.src_extent[d], cons_cfg_x, digits, magic_v, lo, hi);
                uint32_t c = 0;
                if (hi > lo) c = owner_part(hi - 1, e.src_extent[d], cp.deg[d]) - owner_part(lo, e.src_extent[d], cp.deg[d]) + 1;
                n *= c;
            }
        }
    }
    return n;
}

// number of inputs every part of op j waits for (Section 5.1 step 2, counted in closed form)
template <class SimX>
__device__ __forceinline__ uint32_t count_pending(const SimX& m, uint32_t j, const OpCfg& cj) {
    const uint32_t in_begin = m.T.ops[j].in_begin, in_end = m.T.ops[j].in_end;
    const uint32_t digits = part_digits(cj, lane_id(), m.magic_v);
    uint32_t pending = 0;
    for (uint32_t q = in_begin; q < in_end; q++) {
        const DEdge e = m.T.in_edges[q];
        const OpCfg ci = m.cfg(e.src);
        pending += count_inputs<SimX::kTrain>(e, ci, cj.x, digits, m.magic_v);
    }
    return pending;
}

// Section 4: every configuration valid?  Also fills exe_of.  A valid strategy is REGULAR if
// every op puts its parts on consecutive, distinct devices (stride 1, no more parts than
// devices) and a node has at most MAX_RUN GPUs: the event loop has a faster form for those.
enum StrategyClass : uint32_t { STRATEGY_INVALID = 0, STRATEGY_GENERAL = 1, STRATEGY_REGULAR = 2 };
template <class SimX>
__device__ __forceinline__ StrategyClass validate_strategy(const SimX& m) {
    bool bad = false, irregular = false;
    for (uint32_t i = lane_id(); i < m.S.n_ops; i += WAVE) {
        OpCfg c = unpack_cfg_lane(m.cfg_raw(i));
        if (SimX::kExt && m.devmap) c.off = 0;             // offset and stride are not used with explicit devices
        if (!cfg_ok(m.T.ops[i], c, m.S)) {
            bad = true;
        } else if (m.S.n_cols) {
            m.exe_of[i] = m.T.cost[(size_t)i * m.S.n_cols + (c.parts - 1)];
        } else {
            // costs keyed by the whole degree tuple: ptr[n_ops+1], tuples (ascending per op), times;
            // a tuple that is not listed has no cost: invalid
            const uint32_t* ptr = m.T.cost;
            const uint32_t* tuples = ptr + m.S.n_ops + 1;
            const uint32_t* ns = tuples + ptr[m.S.n_ops];
            uint32_t lo = ptr[i], hi = ptr[i + 1];
            while (lo < hi) {
                const uint32_t mid = (lo + hi) / 2;
                if (tuples[mid] < c.x) lo = mid + 1; else hi = mid;
            }
            if (lo < ptr[i + 1] && tuples[lo] == c.x) m.exe_of[i] = ns[lo];
            else bad = true;
        }
        irregular = irregular || c.stride != 1 || c.parts > m.S.n_dev;
        if (SimX::kExt && m.devmap && !bad)
            for (uint32_t k = 0; k < c.parts; k++) bad = bad || m.devmap[(size_t)i * WAVE + k] >= m.S.n_dev;
    }
    if (ballot(bad)) return STRATEGY_INVALID;
    if (SimX::kExt && m.devmap) return STRATEGY_GENERAL;      // the regular form assumes consecutive devices
    return (ballot(irregular) || m.gpn() > MAX_RUN) ? STRATEGY_GENERAL : STRATEGY_REGULAR;
}

}  // namespace ffsim
