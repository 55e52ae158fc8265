// Kernels of the batched execution simulator: one candidate strategy per wavefront.
//
// Task-graph construction (Section 5.1) and Algorithm 1 are fused: the task graph is never
// written out.  A compute task is (op, part); its id is op*64 + part, which is
// order-isomorphic to the dense construction-order id.  Communication tasks are never
// stored: the transfers that start when a producer part finishes are enumerated at that
// moment, one consumer part per lane, and queued on their link rows in
// (edge, producer part, consumer part) order, which is their id order.
//
// The priority queue of Algorithm 1 is a 64-ary min-tree over one 64-bit word per compute
// task (encoding: ffsim_device.h).  Level 0 (the words) lives in HBM, or in LDS for small
// graphs; level 1 (one minimum per op) and level 2 (one per 64 ops) live in LDS.  Popping the
// minimum word and taking the lowest index among equal words reproduces the
// (readyTime, id) order: at equal times, finished producers release their transfers (kind
// 0) before READY compute tasks are dequeued (kind 1); the two kinds never share a device
// row, so only the order inside each kind matters.  All parts of one op that hold the
// minimum word are handled in one step, serialised per device row in lane (= id) order.
#pragma once
#include "ffsim_device.h"

namespace ffsim {

// up to this many groups of 64 ops the queue has no level 2: lanes scan level 1 directly
constexpr uint32_t FLAT_GROUPS = 8;
// GPUs per node up to which transfers are serialised on their link rows by a running sum
// along consecutive lanes (one shift per GPU); beyond, the general search for equal rows runs
constexpr uint32_t MAX_RUN = 8;

// Section timing for development builds (-DFFSIM_PROFILE): shader-clock ticks per section are
// accumulated in a register array and reported through the stats record instead of the
// usual counters.  Compiled out otherwise.
#ifdef FFSIM_PROFILE
#define PROF_DECL u64 prof_t[8] = {cnt.exit_code, 0, 0, 0, 0, 0, 0, 0}; u64 prof_last = __builtin_readcyclecounter();
#define PROF_MARK(k) { const u64 prof_now = __builtin_readcyclecounter(); prof_t[k] += prof_now - prof_last; prof_last = prof_now; }
#define PROF_STORE(c) { c.n_compute = prof_t[0]; c.n_pairs = prof_t[1]; c.n_comm = prof_t[2]; c.sum_comm_ns = lane_id() == 0 ? prof_t[3] : 0; \
                        c.exit_code = prof_t[4]; c.n_stuck = prof_t[5]; c.want_check = prof_t[6]; }
#else
#define PROF_DECL
#define PROF_MARK(k)
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
__host__ __device__ inline size_t ecache_bytes(uint32_t n_edges) { return (size_t)n_edges * 5 * WAVE * 4; }
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

// Serialise tasks that become ready at the same time r on device rows, in lane order
// (= id order): end = max(r, row free time) + running sum of exeTimes on that row.
// One LDS round trip: every lane writes its lane id to a one-byte tag of its row, then reads
// the tag back together with the row's free time.  A lane that reads another lane's id
// shares its row; the lanes of such rows are grouped and ranked with ballots (never through
// memory), everybody else is done at once.  The last lane of every row writes the new free
// time.  `may_share` = false promises distinct rows and skips the tags.
__device__ __forceinline__ u64 fifo_commit(bool act, uint32_t row, u64 exe, u64 r, bool may_share, const WaveLds& L) {
    const int lane = lane_id();
    u64 f = 0;
    bool lost = false;
    if (may_share) {
        if (act) L.tag[row] = (uint8_t)lane;
        wave_sync();
        if (act) { lost = L.tag[row] != (uint8_t)lane; f = L.free_at[row]; }
    } else if (act) {
        f = L.free_at[row];
    }
    const u64 base = f > r ? f : r;         // identical for all lanes of one row
    u64 end = base + exe;
    bool last = act;
    u64 todo = ballot(lost);
    while (todo) {
        const int l = __builtin_ctzll(todo);
        const uint32_t lrow = readlane_u32(row, l);
        const bool peer = act && row == lrow;   // includes the lane whose tag survived
        const u64 peers = ballot(peer);
        todo &= ~peers;
        const int first = __builtin_ctzll(peers);
        const u64 exe_l = readlane_u64(exe, first);
        if (!ballot(peer && exe != exe_l)) {
            // equal exeTimes (symmetric parts): the position in the group is enough
            const uint32_t rank = __builtin_amdgcn_mbcnt_hi((uint32_t)(peers >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)peers, 0u)) + 1;
            if (peer) end = base + (u64)rank * exe;
        } else {
            u64 t = 0;
            u64 pm = peers;
            while (pm) {
                const int p = __builtin_ctzll(pm);
                pm &= pm - 1;
                t += readlane_u64(exe, p);
                if (lane == p) end = base + t;
            }
        }
        if (peer) last = lane == 63 - __builtin_clzll(peers);
    }
    if (last) L.free_at[row] = end;
    wave_sync();
    return end;
}

// Everything one wavefront needs to simulate its candidate.  cfgs is deliberately not
// __restrict__: the chain kernel rewrites a configuration between simulations, so loads
// from it must not be treated as invariant.
// OVR: one op's configuration may be overridden (trial mutations); the plain form does not
// pay for the comparison.
template <bool OVR>
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
    static constexpr bool kOvr = OVR;
    __device__ __forceinline__ uint2 cfg_raw(uint32_t j) const {
        uint2 c = cfgs[j];
        if (OVR && j == ov_op) c = ov_cfg;
        return c;
    }
    __device__ __forceinline__ OpCfg cfg(uint32_t j) const { return unpack_cfg(cfg_raw(j)); }
};
constexpr uint32_t NO_OVERRIDE = 0xffffffffu;
typedef SimT<false> Sim;
typedef SimT<true> SimTrial;

// Optional recording for delta simulation: endTime of every task, and snapshots of the
// simulation state whenever the event time crosses a multiple of `step`.
//
// Every snapshot index has two storage places (set 0 and set 1).  Bit k of `loc` says which of
// them holds snapshot k of the chain's ACCEPTED timeline; a recorded run writes snapshot k into
// the other place, and endTimes into their own array, marked with the run's tag.  Nothing of
// the accepted timeline is touched until the run is committed (the bits of the snapshots it
// wrote are flipped, its endTimes are copied over); a run that is not committed leaves no trace.
struct Recorder {
    u64* end_try;            // [n_ops*64] tag<<48 | endTime of the tasks the run committed (null: not recorded)
    u64* snap_words;         // [2][n_snaps][n_ops*64]
    u64* snap_l1;            // [2][n_snaps][n_ops_pad]
    u64* snap_free;          // [2][n_snaps][n_rows]
    u64 step;                // snapshot k holds the state before the first event with word >= k*step
    u64 tag;                 // this run's tag, already shifted (tag << 48)
    uint32_t loc;            // see above
    uint32_t n_snaps;        // capacity (snapshot 0 is the initial state and is never stored)
    uint32_t next;           // next snapshot index to write
    // Re-convergence: a run that resumed after a change of op check_op compares every state it
    // snapshots (index < check_below) with the accepted timeline's snapshot of the same index.
    // Once they agree (and check_op has no task left), the rest of the two timelines is the same
    // and the run stops.  check_below = 0: no comparison.
    uint32_t check_below;
    uint32_t check_op;
};
constexpr uint32_t MAX_SNAPSHOTS = 32;   // bits of loc
constexpr u64 RUN_CONVERGED = 1;         // run_events: stopped because the timeline re-joined the accepted one

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
#pragma unroll
    for (int d = 0; d < 4; d++) {
        el.nlo[d] = 0; el.nhi[d] = 1;
        if ((uint32_t)d < e.src_ndim) needed_range(e.map[d], e.src_extent[d], cj.x, digits, m.magic_v, el.nlo[d], el.nhi[d]);
    }
    const uint32_t G = S.gpus_per_node;
    // the run fields only depend on the consumer's own configuration: filled whenever it puts its
    // parts on consecutive, distinct devices, whatever the other ops do
    const bool consecutive = cj.stride == 1 && cj.parts <= S.n_dev && G <= MAX_RUN;
    el.dev_c = consecutive ? part_device<true>(cj, lane, S) : part_device<false>(cj, lane, S);
    el.node_c = div_magic(el.dev_c, S.magic_gpn, S.pass_gpn);
    el.pos = 0; el.first_len = 0; el.last_run_mask = 0; el.run_end = false; el.wrapped = false;
    if (consecutive) {
        const uint32_t node0 = div_magic(cj.off, S.magic_gpn, S.pass_gpn);
        const uint32_t room = G - (cj.off - node0 * G);              // lanes of the first run
        el.first_len = cj.parts < room ? cj.parts : room;
        const uint32_t local_c = el.dev_c - el.node_c * G;
        el.pos = (uint32_t)lane < el.first_len ? (uint32_t)lane : local_c;    // index inside the run
        const uint32_t last = cj.off + cj.parts - 1;
        el.wrapped = last >= S.n_dev && div_magic(last - S.n_dev, S.magic_gpn, S.pass_gpn) == node0;
        el.last_run_mask = (el.wrapped && (uint32_t)lane >= el.first_len && el.node_c == node0) ? 0xffffffffu : 0u;
        el.run_end = el.mine && ((uint32_t)lane == cj.parts - 1 || local_c == G - 1) &&
                     !(el.wrapped && (uint32_t)lane == el.first_len - 1);
    }
    return el;
}

// ranges as lo | hi << 16; one word of small fields: device 10 bits, node 10, pos 3, run_end,
// last run, mine, first_len 4, wrapped
__device__ __forceinline__ void ecache_store(uint32_t* ecache, uint32_t eid, const EdgeLane& el) {
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
    return el;
}

// how many parts of the producer (configuration cp) a consumer part reads through edge e:
// the product over the producer's dims of the number of producer parts its range touches
__device__ __forceinline__ uint32_t count_inputs(const DEdge& e, const OpCfg& cp, uint32_t cons_cfg_x, uint32_t digits, uint32_t magic_v) {
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
        pending += count_inputs(e, ci, cj.x, digits, m.magic_v);
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
    }
    if (ballot(bad)) return STRATEGY_INVALID;
    return (ballot(irregular) || m.S.gpus_per_node > MAX_RUN) ? STRATEGY_GENERAL : STRATEGY_REGULAR;
}

template <class SimX>
__device__ __forceinline__ void rebuild_l2(const SimX& m) {
    if (m.S.n_groups > FLAT_GROUPS) {
        for (uint32_t g = 0; g < m.S.n_groups; g++) {
            const u64 wmin = wave_min_u64(m.L.l1[g * WAVE + lane_id()]);
            if (lane_id() == 0) m.L.l2[g] = wmin;
        }
        wave_sync();
    }
}

// Section 5.1 step 1 and the start of Algorithm 1: the tasks, how many inputs each waits
// for, the initial READY set, idle devices.
// the same count from ranges that are already known
__device__ __forceinline__ uint32_t count_inputs_of(const DEdge& e, const OpCfg& cp, const EdgeLane& el) {
    uint32_t n = 1;
#pragma unroll
    for (int d = 0; d < 4; d++) {
        if ((uint32_t)d < e.src_ndim) {
            uint32_t c;
            if (cp.deg[d] == 1) {
                c = el.nhi[d] > el.nlo[d] ? 1u : 0u;           // the producer does not split this dim (uniform)
            } else if (e.map[d].src_dim < 0) {
                c = cp.deg[d];                                   // the whole extent is read: every part (uniform)
            } else {
                c = 0;
                if (el.nhi[d] > el.nlo[d])
                    c = owner_part((uint32_t)el.nhi[d] - 1, e.src_extent[d], cp.deg[d]) - owner_part((uint32_t)el.nlo[d], e.src_extent[d], cp.deg[d]) + 1;
            }
            n *= c;
        }
    }
    return n;
}

template <class SimX>
__device__ __forceinline__ void init_state(SimX& m, Counters& cnt) {
    const int lane = lane_id();
    for (uint32_t r = lane; r < m.S.n_rows; r += WAVE) m.L.free_at[r] = 0;
    for (uint32_t j = 0; j < m.S.n_ops; j++) {
        const OpCfg cj = m.cfg(j);
        uint32_t pending = 0;
        if (m.ecache && m.ecache_fill) {
            // what every later release of an in-edge needs about this op's parts is computed here, once
            const uint32_t in_begin = m.T.ops[j].in_begin, in_end = m.T.ops[j].in_end;
            for (uint32_t q = in_begin; q < in_end; q++) {
                const DEdge e = m.T.in_edges[q];
                const EdgeLane el = edge_lane(m, e, cj);
                ecache_store(m.ecache, e.eid, el);
                pending += count_inputs_of(e, m.cfg(e.src), el);
            }
        } else {
            pending = count_pending(m, j, cj);
        }
        // pending < PENDING_LIMIT is guaranteed by ff_sim_create (at most 511 in-edges per op)
        const u64 w = (uint32_t)lane >= cj.parts ? W_NONE : (pending == 0 ? 1ull : (W_WAIT | ((u64)pending << 48)));
        m.words[j * WAVE + lane] = w;
        // level 1 only has to order pending events: at the start an op has one (READY at time 0) or none
        const u64 any_ready = ballot(w == 1ull);
        if (lane == 0) m.L.l1[j] = any_ready ? 1ull : W_NONE;
        cnt.n_compute += cj.parts;
    }
    for (uint32_t j = m.S.n_ops + lane; j < m.S.n_ops_pad; j += WAVE) m.L.l1[j] = W_NONE;
    wave_sync();
    rebuild_l2(m);
    m.last_key = 0;
    m.overflow = false;
}

// wavefront-wide copy of n 64-bit words between 16-byte aligned HBM buffers, n a multiple of
// 64: 16 bytes per lane and eight loads in flight before the first store
__device__ __forceinline__ void copy_words(u64* __restrict__ dst, const u64* __restrict__ src, uint32_t n) {
    const uint4* __restrict__ s4 = (const uint4*)src;
    uint4* __restrict__ d4 = (uint4*)dst;
    const uint32_t n4 = n / 2;          // multiple of 32
    uint32_t t = lane_id();
    for (; t + 7 * WAVE < n4; t += 8 * WAVE) {
        uint4 v[8];
#pragma unroll
        for (int u = 0; u < 8; u++) v[u] = s4[t + u * WAVE];
#pragma unroll
        for (int u = 0; u < 8; u++) d4[t + u * WAVE] = v[u];
    }
    for (; t < n4; t += WAVE) d4[t] = s4[t];
}

// the same copy, and: does src differ from old anywhere?  (per lane; combine with a ballot)
__device__ __forceinline__ bool copy_words_compare(u64* __restrict__ dst, const u64* __restrict__ src, const u64* __restrict__ old,
                                                   uint32_t n) {
    const uint4* __restrict__ s4 = (const uint4*)src;
    const uint4* __restrict__ o4 = (const uint4*)old;
    uint4* __restrict__ d4 = (uint4*)dst;
    const uint32_t n4 = n / 2;
    uint32_t diff = 0;
    uint32_t t = lane_id();
    for (; t + 3 * WAVE < n4; t += 4 * WAVE) {
        uint4 v[4], o[4];
#pragma unroll
        for (int u = 0; u < 4; u++) { v[u] = s4[t + u * WAVE]; o[u] = o4[t + u * WAVE]; }
#pragma unroll
        for (int u = 0; u < 4; u++) {
            d4[t + u * WAVE] = v[u];
            diff |= (v[u].x ^ o[u].x) | (v[u].y ^ o[u].y) | (v[u].z ^ o[u].z) | (v[u].w ^ o[u].w);
        }
    }
    for (; t < n4; t += WAVE) {
        const uint4 v = s4[t], o = o4[t];
        d4[t] = v;
        diff |= (v.x ^ o.x) | (v.y ^ o.y) | (v.z ^ o.z) | (v.w ^ o.w);
    }
    return diff != 0;
}

// Writes the next snapshot.  Returns true if the comparison is on and the state equals the
// accepted timeline's snapshot of the same index for everything that can still matter: all task
// words, and the free time of every device row, where rows that are idle at the snapshot's
// time count as equal (any later task is ready at or after that time).
template <class SimX>
__device__ __forceinline__ bool save_snapshot(const SimX& m, Recorder& rec) {
    const int lane = lane_id();
    const uint32_t idx = rec.next;
    const size_t k = (size_t)((((rec.loc >> idx) & 1u) ^ 1u) * rec.n_snaps + idx);   // the place the accepted timeline does not use
    const bool check = idx < rec.check_below;
    bool differs = false;
    const size_t nw = (size_t)m.S.n_ops * WAVE;
    if (check) {
        const size_t old = (size_t)(((rec.loc >> idx) & 1u) * rec.n_snaps + idx);
        differs = copy_words_compare(rec.snap_words + k * nw, m.words, rec.snap_words + old * nw, m.S.n_ops * WAVE);
        const u64 t_snap = ((u64)idx * rec.step) >> 1;
        const u64* ofr = rec.snap_free + old * (size_t)m.S.n_rows;
        for (uint32_t t = lane; t < m.S.n_rows; t += WAVE) {
            const u64 a = m.L.free_at[t], b = ofr[t];
            differs = differs || (a > t_snap ? a : t_snap) != (b > t_snap ? b : t_snap);
        }
        // a task of the changed op still pending would make equal words mean different things
        differs = differs || m.words[(size_t)rec.check_op * WAVE + lane] != W_NONE;
    } else {
        copy_words(rec.snap_words + k * nw, m.words, m.S.n_ops * WAVE);
    }
    u64* l1 = rec.snap_l1 + k * (size_t)m.S.n_ops_pad;
    for (uint32_t t = lane; t < m.S.n_ops_pad; t += WAVE) l1[t] = m.L.l1[t];
    u64* fr = rec.snap_free + k * (size_t)m.S.n_rows;
    for (uint32_t t = lane; t < m.S.n_rows; t += WAVE) fr[t] = m.L.free_at[t];
    rec.next++;
    return check && !ballot(differs);
}

// snapshot k of the accepted timeline
template <class SimX>
__device__ __forceinline__ void load_snapshot(SimX& m, const Recorder& rec, uint32_t k) {
    const int lane = lane_id();
    const size_t at = (size_t)(((rec.loc >> k) & 1u) * rec.n_snaps + k);
    copy_words(m.words, rec.snap_words + at * m.S.n_ops * WAVE, m.S.n_ops * WAVE);
    const u64* l1 = rec.snap_l1 + at * m.S.n_ops_pad;
    for (uint32_t t = lane; t < m.S.n_ops_pad; t += WAVE) m.L.l1[t] = l1[t];
    const u64* fr = rec.snap_free + at * m.S.n_rows;
    for (uint32_t t = lane; t < m.S.n_rows; t += WAVE) m.L.free_at[t] = fr[t];
    wave_sync();
    m.last_key = (u64)k * rec.step;
    m.overflow = false;
}

// Algorithm 1, main loop, from the current state to the end.  RECORD: keep endTimes and
// snapshots for delta simulation.  Returns 0 or a RESULT_* code.
// REG: the strategy is STRATEGY_REGULAR.  STATS: also count pairs and transfers (the optional
// per-candidate record); a compile-time switch so that the counters cost the timed path nothing.
// CACHE: the per-edge set-up was stored by init_state (m.ecache).
// Q: shape of the queue above the task words.
//   Q_ONE   at most 64 ops: level 1 (one minimum per op) sits in a register, lane = op; nothing of
//           the queue is in LDS while the loop runs (batch kernels only: level 1 is not written back);
//   Q_FLAT  up to FLAT_GROUPS groups of 64 ops: level 1 in LDS, every lane scans its column;
//   Q_TREE  more groups: level 1 in LDS, level 2 (one minimum per group) in a register, lane = group.
enum QueueShape : int { Q_ONE = 0, Q_FLAT = 1, Q_TREE = 2 };
template <bool WIDE, bool RECORD, bool REG, bool STATS, int Q, bool CACHE, class SimX>
__device__ u64 run_events(SimX& m, Counters& cnt, Recorder& rec) {
    constexpr bool TREE = Q == Q_TREE;
    const int lane = lane_id();
    PROF_DECL
    const SimDev& S = m.S;
    const WaveLds& L = m.L;
    const DOp* __restrict__ ops = m.T.ops;
    const DEdge* __restrict__ edges = m.T.edges;
    u64* words = m.words;
    const uint32_t magic_v = m.magic_v;
    u64 last_key = m.last_key;
    bool overflow = m.overflow;
    // the register-resident level of the queue (see QueueShape)
    u64 qreg = W_NONE;
    if (Q == Q_ONE) qreg = L.l1[lane];
    if (Q == Q_TREE) qreg = (uint32_t)lane < S.n_groups ? L.l2[lane] : W_NONE;
    // Values chosen per lane between two of these (same node or not) must sit in registers: a
    // select between two fields of the argument block is otherwise turned into a per-lane load
    // from that block, a vector memory round trip for every producer part.
    const uint32_t bw_intra = first_u32(S.bw_intra), bw_inter = first_u32(S.bw_inter);
    const uint32_t m_bw_intra = first_u32(S.m_bw_intra), m_bw_inter = first_u32(S.m_bw_inter);
    const uint32_t lat_intra = first_u32(S.lat_intra), lat_inter = first_u32(S.lat_inter);
    const u64 max_events = 2ull * S.n_ops * WAVE + 8;   // every task is popped at most twice
    for (u64 ev = 0; ev < max_events; ev++) {
        u64 kmin;
        uint32_t i;
        if (Q == Q_ONE) {
            kmin = wave_min_from(qreg, last_key);
            if (kmin >> 63) break;
            const u64 m1 = ballot(qreg == kmin);
            if (!m1) { cnt.exit_code = 1; return RESULT_INTERNAL; }
            i = __builtin_ctzll(m1);                 // lowest op index among equal keys
        } else if (TREE) {
            const u64 k2 = qreg;
            kmin = wave_min_from(k2, last_key);
            if (kmin >> 63) break;
            const uint32_t g = __builtin_ctzll(ballot(k2 == kmin));
            const u64 k1 = L.l1[g * WAVE + lane];
            const u64 m1 = ballot(k1 == kmin);
            if (!m1) { cnt.exit_code = 1; return RESULT_INTERNAL; }   // tree inconsistent: give up, never spin
            i = g * WAVE + __builtin_ctzll(m1);
        } else {
            // few ops: every lane scans its column of level 1, no level 2
            u64 k1 = L.l1[lane];
            uint32_t gbest = 0;
            for (uint32_t g = 1; g < S.n_groups; g++) {
                const u64 k = L.l1[g * WAVE + lane];
                if (k < k1) { k1 = k; gbest = g; }
            }
            kmin = wave_min_from(k1, last_key);
            if (kmin >> 63) break;
            // lowest op index among equal keys: smallest group first, then lowest lane
            u64 m1 = ballot(k1 == kmin);
            if (!m1) { cnt.exit_code = 1; return RESULT_INTERNAL; }
            if (m1 & (m1 - 1)) {    // several columns hold the minimum: smallest group wins
                const uint32_t gmin = wave_min_u32(k1 == kmin ? gbest : 0xffffffffu);
                m1 = ballot(k1 == kmin && gbest == gmin);
            }
            const int col = __builtin_ctzll(m1);
            i = readlane_u32(gbest, col) * WAVE + col;
        }
        static_assert(!(RECORD && Q == Q_ONE), "snapshots read level 1 from LDS");
        if (RECORD) {
            // the state before the first event at or after a multiple of `step` is a snapshot
            while (rec.next < rec.n_snaps && kmin >= (u64)rec.next * rec.step) {
                if (save_snapshot(m, rec)) { m.last_key = last_key; return RUN_CONVERGED; }
            }
        }
        last_key = kmin;
        PROF_MARK(1)
        // everything that depends only on i is requested together
        u64 k0 = words[i * WAVE + lane];
        const DOp* __restrict__ opi_p = ops + i;
        const uint32_t out_begin = opi_p->out_begin, out_end = opi_p->out_end;
        const OpCfg ci = m.cfg(i);
        const u64 exe = m.exe_of[i];
        const u64 mask = ballot(k0 == kmin);            // parts of op i that hold the minimum
        if (!mask) { cnt.exit_code = 2; return RESULT_INTERNAL; }
        cnt.n_events++;
        const u64 now = kmin >> 1;
        const bool in_mask = (mask >> lane) & 1;
        const uint32_t dev_p = part_device<REG>(ci, lane, S);

        if (kmin & 1) {
            // dequeue READY compute tasks: start = max(readyTime, device free), end = start + exeTime
            const bool may_share = REG ? false : !(ci.stride == 1 && ci.parts <= S.n_dev);
            const u64 end = fifo_commit(in_mask, dev_p, exe, now, may_share, L);
            overflow = overflow || end >= TIME_LIMIT;
            if (in_mask) k0 = out_end > out_begin ? end << 1 : W_NONE;
            if (RECORD) { if (in_mask && rec.end_try) rec.end_try[i * WAVE + lane] = rec.tag | end; }
            PROF_MARK(2)
        } else {
            // the parts in `mask` finished at `now`: release their successors edge by edge
            DEdge e = opi_p->first;
            const Box pb = part_box(e.src_extent, ci, lane, magic_v);
            const uint32_t node_p = div_magic(dev_p, S.magic_gpn, S.pass_gpn);
            for (uint32_t ei = out_begin; ei < out_end; ei++) {
                if (ei != out_begin) e = edges[ei];
                const uint32_t j = e.dst;
                u64 w = words[j * WAVE + lane];
                // REG: consumer parts sit on consecutive, distinct devices, so the transfers from
                // one producer part can share a link row only when their consumers sit on the
                // same remote node, and those consumers are a run of consecutive lanes (the node
                // of lane 0 may come back once more at the end, after the device numbers wrapped
                // around).  The FIFO order on every shared row is then a running sum along the
                // run, and no search for lanes with equal rows is needed.
                // (the op of a trial mutation differs from what the chain's kept set-up describes)
                const EdgeLane el = (CACHE && !(SimX::kOvr && j == m.ov_op)) ? ecache_load(m.ecache, ei) : edge_lane(m, e, m.cfg(j));
                const bool mine = el.mine;
                int32_t nlo[4], nhi[4];
#pragma unroll
                for (int d = 0; d < 4; d++) { nlo[d] = el.nlo[d]; nhi[d] = el.nhi[d]; }
                const uint32_t dev_c = el.dev_c, node_c = el.node_c;
                const uint32_t local_c = dev_c - node_c * S.gpus_per_node;
                const uint32_t G = S.gpus_per_node;
                const uint32_t pos = el.pos, first_len = el.first_len, last_run_mask = el.last_run_mask;
                const bool run_end = el.run_end, wrapped = el.wrapped;
                u64 ready = w & (TIME_LIMIT - 1);
                uint32_t pending = (uint32_t)(w >> 48) & PENDING_LIMIT;
                bool touched = false;
                u64 todo = mask;
                PROF_MARK(3)
                while (todo) {
                    const int kp = __builtin_ctzll(todo);
                    todo &= todo - 1;
                    bool hit = mine;
                    u64 elems = 1;
#pragma unroll
                    for (int d = 0; d < 4; d++) {
                        if ((uint32_t)d < e.src_ndim) {
                            const int32_t plo = (int32_t)readlane_u32(pb.lo[d], kp), phi = (int32_t)readlane_u32(pb.hi[d], kp);
                            const int32_t lo = nlo[d] > plo ? nlo[d] : plo;
                            const int32_t hi = nhi[d] < phi ? nhi[d] : phi;
                            hit = hit && hi > lo;
                            if (WIDE) elems *= (u64)(uint32_t)(hi > lo ? hi - lo : 0);
                            else elems = (uint32_t)elems * (uint32_t)(hi > lo ? hi - lo : 0);
                        }
                    }
                    const u64 hit_mask = ballot(hit);
                    if (!hit_mask) continue;
                    const uint32_t dev_a = readlane_u32(dev_p, kp);
                    const uint32_t node_a = readlane_u32(node_p, kp);
                    const bool comm = hit && dev_c != dev_a;
                    const u64 comm_mask = ballot(comm);
                    u64 arrive = now;
                    if (comm_mask) {
                        const bool same_node = node_c == node_a;
                        // Section 5.1: the link device between the two devices.  The producer's share of
                        // the row index is scalar; per lane one select between two sums.
                        const uint32_t row_intra = S.n_dev + node_a * G * G + (dev_a - node_a * G) * G;
                        const uint32_t row_inter = S.n_dev + S.n_nodes * G * G + node_a * S.n_nodes;
                        const uint32_t to_intra = row_intra + local_c, to_inter = row_inter + node_c;
                        const uint32_t row = same_node ? to_intra : to_inter;
                        // assumption A2: transfer time = size / bandwidth (rounded up) + latency
                        const uint32_t bw = same_node ? bw_intra : bw_inter;
                        u64 ns;
                        if (WIDE) {
                            const u64 bytes = elems * S.elem_bytes;
                            ns = (bytes + bw - 1) / bw;
                        } else {
                            const uint32_t bytes = (uint32_t)elems * S.elem_bytes;
                            ns = ceil_div_u32(comm ? bytes : 1u, bw, same_node ? m_bw_intra : m_bw_inter);
                        }
                        ns += same_node ? lat_intra : lat_inter;
                        u64 end;
                        if (REG) {
                            const u64 f = L.free_at[row];                  // in range for every lane
                            const u64 base = f > now ? f : now;            // the same for all lanes of a row
                            const bool chained = comm && !same_node;       // rows between GPUs of one node are private
                            u64 incl;
                            if (!WIDE) {
                                // a row's running sum of transfer times cannot reach 2^32 (the host
                                // selects the WIDE kernels otherwise)
                                uint32_t acc = chained ? (uint32_t)ns : 0u, t = acc;
                                for (uint32_t sft = 1; sft < G; sft++) {
                                    t = wave_shr1_u32(t);
                                    if (pos < sft) t = 0;
                                    acc += t;
                                }
                                if (wrapped) acc += readlane_u32(acc, (int)first_len - 1) & last_run_mask;
                                incl = acc;
                            } else {
                                u64 t = incl = chained ? ns : 0;
                                for (uint32_t sft = 1; sft < G; sft++) {
                                    t = wave_shr1_u64(t);
                                    if (pos < sft) t = 0;
                                    incl += t;
                                }
                                if (wrapped) {
                                    const u64 first_total = readlane_u64(incl, (int)first_len - 1);
                                    if (last_run_mask) incl += first_total;
                                }
                            }
                            end = base + (same_node ? ns : incl);
                            if (same_node ? comm : (run_end && incl != 0)) L.free_at[row] = end;
                            wave_sync();
                        } else {
                            end = fifo_commit(comm, row, ns, now, true, L);
                        }
                        if (comm) arrive = end;
                        if (STATS) {
                            cnt.n_comm += __popcll(comm_mask);
                            if (comm) cnt.sum_comm_ns += ns;   // per-lane partial sums, reduced by the caller
                        }
                    }
                    if (hit) {
                        ready = arrive > ready ? arrive : ready;
                        pending -= 1;
                        touched = true;
                    }
                    if (STATS) cnt.n_pairs += __popcll(hit_mask);
                }
                PROF_MARK(4)
                overflow = overflow || (touched && ready >= TIME_LIMIT);
                const bool now_ready = touched && pending == 0;
                if (touched) {
                    w = now_ready ? ((ready << 1) | 1) : (W_WAIT | ((u64)pending << 48) | (ready & (TIME_LIMIT - 1)));
                    words[j * WAVE + lane] = w;
                }
                if (ballot(now_ready)) {
                    const u64 nmin = wave_min_from(now_ready ? w : W_NONE, last_key);
                    if (Q == Q_ONE) {
                        if ((uint32_t)lane == j && nmin < qreg) qreg = nmin;
                    } else {
                        if (lane == 0 && nmin < L.l1[j]) L.l1[j] = nmin;
                        if (TREE && (uint32_t)lane == (j >> 6) && nmin < qreg) qreg = nmin;
                    }
                }
                PROF_MARK(5)
            }
            if (in_mask) k0 = W_NONE;
        }
        if (in_mask) words[i * WAVE + lane] = k0;
        const u64 new_l1 = wave_min_from(k0, last_key);
        if (Q == Q_ONE) {
            if ((uint32_t)lane == i) qreg = new_l1;
            wave_sync();
        } else {
            wave_sync();
            if (lane == 0) L.l1[i] = new_l1;
            wave_sync();
        }
        if (TREE) {
            const uint32_t g = i >> 6;
            const u64 new_l2 = wave_min_from(L.l1[g * WAVE + lane], last_key);
            if ((uint32_t)lane == g) qreg = new_l2;
        }
        PROF_MARK(6)
    }
    m.last_key = last_key;
    PROF_STORE(cnt)
    if (ballot(overflow)) return RESULT_OVERFLOW;
    return 0;
}

// Algorithm 1, result (largest endTime): every transfer feeds a compute task that ends
// later, so the makespan is the largest free time over the compute device rows.
template <class SimX>
__device__ __forceinline__ u64 makespan(const SimX& m) {
    u64 mk = 0;
    for (uint32_t d = lane_id(); d < m.S.n_dev; d += WAVE) mk = m.L.free_at[d] > mk ? m.L.free_at[d] : mk;
    return wave_max_u64(mk);
}

// One candidate: build + simulate.  Returns the makespan or one of the RESULT_* codes.
// WIDE selects 64-bit element counts (tensors of 2^32 bytes or more).
template <bool WIDE, bool RECORD, bool STATS, int Q, bool CACHE>
__device__ u64 simulate_candidate(Sim& m, Counters& cnt, Recorder& rec) {
#ifdef FFSIM_PROFILE
    const u64 prof_t0 = __builtin_readcyclecounter();
#endif
    const StrategyClass cls = validate_strategy(m);
    if (cls == STRATEGY_INVALID) return RESULT_INVALID;
    init_state(m, cnt);
#ifdef FFSIM_PROFILE
    cnt.exit_code = __builtin_readcyclecounter() - prof_t0;   // reported as section 0
#endif
    const u64 rc = cls == STRATEGY_REGULAR ? run_events<WIDE, RECORD, true, STATS, Q, CACHE>(m, cnt, rec)
                                            : run_events<WIDE, RECORD, false, STATS, Q, CACHE>(m, cnt, rec);
    if (rc) return rc;
    if (STATS) {   // diagnostics: tasks that never ran (0 in a correct run)
        for (uint32_t j = 0; j < m.S.n_ops; j++) cnt.n_stuck += __popcll(ballot(m.words[j * WAVE + lane_id()] != W_NONE));
    }
    return makespan(m);
}

__device__ __forceinline__ void store_counters(Counters c, Counters* out) {
    u64 s = c.sum_comm_ns;   // accumulated per lane
#pragma unroll
    for (int k = 1; k < WAVE; k <<= 1) s += shfl_xor_u64(s, k);
    c.sum_comm_ns = s;
    if (lane_id() == 0) *out = c;
}

// lane l gets the multiply-high constant of the divisor l+1
__device__ __forceinline__ uint32_t load_magic(const uint32_t* __restrict__ magic) { return magic[lane_id() + 1]; }

// LDSW: the task words and per-op exeTimes of the candidate live in LDS (small graphs).
// CACHE: the per-edge set-up is kept (after the task words: in LDS if LDSW, else in the slot).
template <bool WIDE, bool LDSW, bool STATS, int Q, bool CACHE>
__global__ __launch_bounds__(WAVE) void k_sim_batch(SimDev S, const DOp* __restrict__ ops, const DEdge* __restrict__ edges,
                                                    const DEdge* __restrict__ in_edges, const uint32_t* __restrict__ cost,
                                                    const uint32_t* __restrict__ magic, const uint2* __restrict__ strategies,
                                                    uint32_t B, u64* __restrict__ out_ns, Counters* __restrict__ stats,
                                                    unsigned char* __restrict__ ws, size_t slot_stride) {
    extern __shared__ __align__(16) unsigned char lds_raw[];
    const Tables T{ops, edges, in_edges, cost};
    u64* words;
    uint32_t* exe_of;
    uint32_t* ecache = nullptr;
    unsigned char* lds_rest = lds_raw;
    const size_t state_bytes = (slot_bytes(S.n_ops, S.n_ops_pad) + 15) & ~(size_t)15;
    if (LDSW) {
        words = (u64*)lds_raw;
        exe_of = (uint32_t*)(lds_raw + (size_t)S.n_ops * WAVE * 8);
        lds_rest = lds_raw + state_bytes;
        if (CACHE) { ecache = (uint32_t*)lds_rest; lds_rest += ecache_bytes(S.n_edges); }
    } else {
        unsigned char* slot = ws + (size_t)blockIdx.x * slot_stride;
        words = (u64*)slot;
        exe_of = (uint32_t*)(slot + (size_t)S.n_ops * WAVE * 8);
        if (CACHE) ecache = (uint32_t*)(slot + state_bytes);
    }
    const WaveLds L = carve_lds(lds_rest, S);
    const uint32_t magic_v = load_magic(magic);
    Recorder none = {};
    for (uint32_t b = blockIdx.x; b < B; b += gridDim.x) {
        Counters cnt = {};
        Sim m{S, T, strategies + (size_t)b * S.n_ops, words, exe_of, L, magic_v, 0, false, NO_OVERRIDE, make_uint2(0, 0), ecache, true};
        const u64 mk = simulate_candidate<WIDE, false, STATS, Q, CACHE>(m, cnt, none);
        if (lane_id() == 0) out_ns[b] = mk;
        if (STATS) store_counters(cnt, stats + b);
        wave_sync();
    }
}

// ---- delta simulation (Section 5.3) ---------------------------------------------------
//
// A chain keeps, in HBM, its current strategy, the endTime of every task of the simulation of
// that strategy (the accepted timeline) and up to n_snaps snapshots of the simulation state
// taken whenever the event time crossed a multiple of `step`.  When the configuration of one
// op changes, nothing can differ before the first producer of that op finishes (its transfers
// are the first tasks that depend on the op's configuration), so the simulation is resumed
// from the last snapshot before that time: the op's own tasks are rebuilt, the input counts of
// its consumers are corrected, and Algorithm 1 continues from there.  The resulting timeline is
// the one a full simulation produces.  Every such run is recorded beside the accepted timeline
// (see Recorder) and becomes the accepted one only when it is committed, so a search proposal
// costs one resumed simulation whether it is accepted or not.
struct ChainMeta {
    u64 step;           // event-word distance between snapshots (2 * time)
    uint32_t n_valid;   // snapshots 1..n_valid-1 are usable (0 = none; index 0 is the initial state)
    uint32_t stale;     // the stored timeline does not belong to the current strategy
    // telemetry (ff_sim_chains_get_stats)
    u64 n_steps;        // mutations applied
    u64 n_resumed;      // of those, resumed from a snapshot instead of simulated from time 0
    u64 n_events;       // queue pops spent in mutation steps
    u64 n_events_full;  // queue pops of the last simulation from time 0 (one full simulation)
    u64 cur_ns;         // simulated time of the chain's current strategy (result code if it has none)
    u64 idle_steps;     // search steps since the chain's best time last improved
    u64 n_converged;    // committed steps whose run stopped early because it re-joined the accepted timeline
    uint32_t loc;       // bit k: which of its two places holds snapshot k of the accepted timeline
    uint32_t tag;       // tag of the last recorded run (1..0xffff; 0 marks entries never written)
};

struct ChainMem {       // all pointers are per chain
    uint2* cfgs;
    u64* words;
    uint32_t* exe_of;
    u64* end_of;        // accepted timeline
    u64* end_try;       // tag<<48 | endTime, written by recorded runs
    u64* snap_words;    // [2][n_snaps][n_ops*64]
    u64* snap_l1;       // [2][n_snaps][n_ops_pad]
    u64* snap_free;     // [2][n_snaps][n_rows, padded to even]
    uint32_t* ecache;   // kept per-edge set-up of the chain's current strategy (see EdgeLane)
    ChainMeta* meta;
};

// byte offset of the ChainMeta record inside a chain block (it comes last)
__host__ __device__ inline size_t chain_meta_offset(uint32_t n_ops, uint32_t n_ops_pad, uint32_t n_rows, uint32_t n_snaps,
                                                    uint32_t n_edges) {
    size_t b = (size_t)n_ops_pad * 8;                       // cfgs
    b += ecache_bytes(n_edges);
    b += (size_t)n_ops * WAVE * 8 * 3;                      // words, end_of, end_try
    b += 2 * (size_t)n_snaps * ((size_t)n_ops * WAVE * 8 + (size_t)n_ops_pad * 8 + (size_t)((n_rows + 1) & ~1u) * 8);
    b += (size_t)n_ops_pad * 4;                             // exe_of
    return b;
}
__host__ __device__ inline size_t chain_bytes(uint32_t n_ops, uint32_t n_ops_pad, uint32_t n_rows, uint32_t n_snaps, uint32_t n_edges) {
    return (chain_meta_offset(n_ops, n_ops_pad, n_rows, n_snaps, n_edges) + sizeof(ChainMeta) + 255) & ~(size_t)255;
}

__device__ __forceinline__ ChainMem carve_chain(unsigned char* base, const SimDev& S, uint32_t n_snaps) {
    ChainMem c;
    const size_t nw = (size_t)S.n_ops * WAVE;
    c.cfgs = (uint2*)base; base += (size_t)S.n_ops_pad * 8;
    c.ecache = (uint32_t*)base; base += ecache_bytes(S.n_edges);
    c.words = (u64*)base; base += nw * 8;
    c.end_of = (u64*)base; base += nw * 8;
    c.end_try = (u64*)base; base += nw * 8;
    c.snap_words = (u64*)base; base += 2 * (size_t)n_snaps * nw * 8;
    c.snap_l1 = (u64*)base; base += 2 * (size_t)n_snaps * S.n_ops_pad * 8;
    c.snap_free = (u64*)base; base += 2 * (size_t)n_snaps * ((S.n_rows + 1) & ~1u) * 8;
    c.exe_of = (uint32_t*)base; base += (size_t)S.n_ops_pad * 4;
    c.meta = (ChainMeta*)base;
    return c;
}

// Where may a simulation start after op `mo` went from configuration `ocfg` to the one now
// in m.cfgs?  Nothing can differ before the first task of a producer of op mo finishes (the
// transfers released then are the first tasks that depend on op mo's configuration); time 0
// if op mo has no producer or has a part without inputs.  Returns the index of the last
// snapshot at or before that time (0 = start from time 0) and, in pend_new, the number of
// inputs every part of op mo waits for under the new configuration.
template <class SimX>
__device__ __forceinline__ uint32_t resume_point(const SimX& m, const u64* end_of, const ChainMeta& meta, uint32_t mo, uint2 ocfg,
                                                 uint32_t& pend_new) {
    const int lane = lane_id();
    const OpCfg cn = m.cfg(mo);
    const OpCfg co = unpack_cfg(ocfg);
    const uint32_t in_begin = m.T.ops[mo].in_begin, in_end = m.T.ops[mo].in_end;
    u64 tau = in_end > in_begin ? W_NONE : 0;
    for (uint32_t q = in_begin; q < in_end; q++) {
        const uint32_t p = m.T.in_edges[q].src;
        const OpCfg cp = m.cfg(p);
        const u64 t = wave_min_u64((uint32_t)lane < cp.parts ? end_of[p * WAVE + lane] : W_NONE);
        tau = t < tau ? t : tau;
    }
    pend_new = count_pending(m, mo, cn);
    uint32_t pend_old = 0;
    {
        const uint32_t digits = part_digits(co, lane, m.magic_v);
        for (uint32_t q = in_begin; q < in_end; q++) {
            const DEdge e = m.T.in_edges[q];
            pend_old += count_inputs(e, m.cfg(e.src), co.x, digits, m.magic_v);
        }
    }
    if (ballot(((uint32_t)lane < cn.parts && pend_new == 0) || ((uint32_t)lane < co.parts && pend_old == 0))) tau = 0;
    u64 k64 = (2 * tau) / meta.step;
    if (k64 > meta.n_valid - 1) k64 = meta.n_valid - 1;
    return (uint32_t)k64;
}

// A simulation state taken before anything depended on op mo's configuration holds two static
// things about it: the op's own tasks (all still waiting for all their inputs) and, in its
// consumers' waiting tasks, how many inputs come from op mo.  Rewrites both for the new
// configuration.  words / l1: the state to patch (a stored snapshot, or live state).
template <class SimX>
__device__ __forceinline__ void patch_state_for_op(const SimX& m, u64* words, u64* l1, uint32_t mo, uint2 ocfg, uint32_t pend_new) {
    const int lane = lane_id();
    const OpCfg cn = m.cfg(mo);
    const OpCfg co = unpack_cfg(ocfg);
    const u64 w_own = (uint32_t)lane >= cn.parts ? W_NONE : (W_WAIT | ((u64)pend_new << 48));
    words[mo * WAVE + lane] = w_own;
    const u64 w_own_min = wave_min_u64(w_own);
    if (lane == 0) l1[mo] = w_own_min;
    const uint32_t ob = m.T.ops[mo].out_begin, oe = m.T.ops[mo].out_end;
    for (uint32_t ei = ob; ei < oe; ei++) {
        const DEdge e = m.T.edges[ei];
        const uint32_t j = e.dst;
        const OpCfg cj = m.cfg(j);
        const uint32_t digits = part_digits(cj, lane, m.magic_v);
        const uint32_t was = count_inputs(e, co, cj.x, digits, m.magic_v);
        const uint32_t is = count_inputs(e, cn, cj.x, digits, m.magic_v);
        if (!ballot((uint32_t)lane < cj.parts && was != is)) continue;
        const u64 w = words[j * WAVE + lane];
        // a part of op j that reads op mo at all is still waiting in such a state
        const bool waiting = (uint32_t)lane < cj.parts && (w >> 63) && w != W_NONE;
        if (waiting && was != is) {
            const uint32_t pending = ((uint32_t)(w >> 48) & PENDING_LIMIT) - was + is;
            words[j * WAVE + lane] = W_WAIT | ((u64)pending << 48) | (w & (TIME_LIMIT - 1));
        }
        // level 1 of op j is unaffected: waiting words are not events
    }
}

// ---- search (Section 6): proposals and Metropolis acceptance, all in integers ------------
//
// Counter-based draws: SplitMix64's finaliser chained over (seed, purpose, chain, step), the
// same generator the input generators use, so a host reference can reproduce every decision.
__device__ __forceinline__ u64 mix64(u64 x) {
    x += 0x9E3779B97F4A7C15ull;
    x = (x ^ (x >> 30)) * 0xBF58476D1CE4E5B9ull;
    x = (x ^ (x >> 27)) * 0x94D049BB133111EBull;
    return x ^ (x >> 31);
}
__device__ __forceinline__ u64 draw64(u64 seed, u64 purpose, u64 chain, u64 step) {
    const u64 K = 0xD6E8FEB86659FD93ull;
    u64 h = mix64(seed);
    h = mix64(h ^ (purpose * K));
    h = mix64(h ^ (chain * K));
    h = mix64(h ^ (step * K));
    return h;
}

// what ff_sim_search hands to the kernel (device pointers)
struct SearchDev {
    u64 seed;
    u64 first_step;              // draws use first_step + s, so that consecutive calls continue one sequence
    u64 bucket_ns;               // width of an acceptance bucket
    const uint32_t* accept;      // [n_buckets] acceptance probability * 2^32 for a proposal worse by that bucket
    const uint32_t* tuple_ptr;   // [n_ops+1] ranges into tuples[]
    const uint32_t* tuples;      // degree tuples (four bytes each) a proposal may pick for each op
    uint32_t n_buckets;
    uint32_t enabled;
    u64 patience;                // a chain stops proposing after this many steps without a new best (0 = never)
    u64* best_ns;                // [C] best simulated time seen (in/out)
    uint2* best_cfgs;            // [C][n_ops] the strategy that achieved it (in/out)
};

// the kept set-up of op j's in-edges follows its configuration
template <class SimX>
__device__ __forceinline__ void refresh_ecache_for_op(const SimX& m, uint32_t j) {
    const OpCfg cj = m.cfg(j);
    const uint32_t in_begin = m.T.ops[j].in_begin, in_end = m.T.ops[j].in_end;
    for (uint32_t q = in_begin; q < in_end; q++) {
        const DEdge e = m.T.in_edges[q];
        ecache_store(m.ecache, e.eid, edge_lane(m, e, cj));
    }
    __threadfence_block();
    wave_sync();
}

// Makes a recorded run the chain's accepted timeline: the snapshots it wrote (first..next-1)
// take the place of the old ones, the endTimes it wrote are copied over the old ones.
// converged: the run stopped where it re-joined the accepted timeline, whose later snapshots and
// endTimes stay.
__device__ __forceinline__ void commit_run(const ChainMem& cm, ChainMeta& meta, const Recorder& rec, uint32_t first, uint32_t n_words,
                                           bool converged) {
    const uint32_t written = rec.next > first ? (uint32_t)(((1ull << rec.next) - 1) & ~((1ull << first) - 1)) : 0u;
    meta.loc ^= written;
    if (!converged) meta.n_valid = rec.next;
    const u64 tag = rec.tag;
    for (uint32_t t = lane_id(); t < n_words; t += WAVE) {
        const u64 v = cm.end_try[t];
        if ((v & ~(TIME_LIMIT - 1)) == tag) cm.end_of[t] = v & (TIME_LIMIT - 1);
    }
    __threadfence_block();
    wave_sync();
}

// One kernel drives a chain through a sequence of steps.  Three sources of steps:
//   muts == nullptr and no search: simulate the chain's starting strategy (n_steps is 1);
//   muts: forced mutations, [n_steps][C] records {op, cfg.x, cfg.y}, always committed;
//   search: per step one proposal (random op, random configuration from its list, random
//           device offset), committed if it is not slower, else with the tabulated probability.
// A step is one recorded simulation (resumed from the last snapshot before the change can
// matter), then either commit_run or nothing.  Every simulation goes through the single
// run_events call site below, including the pass that only finds the makespan when no
// snapshot spacing is set yet.
// A forced mutation that names an op outside the graph poisons the chain: this and all
// later results are RESULT_INVALID.  out_ns[s][c] is the time of the chain's strategy after
// step s.
// CACHE: the chain keeps the per-edge set-up of its current strategy (all extents fit 16 bits).
template <bool WIDE, bool TREE, bool CACHE>
__global__ __launch_bounds__(WAVE) void k_sim_chain_steps(SimDev S, const DOp* __restrict__ ops, const DEdge* __restrict__ edges,
                                                          const DEdge* __restrict__ in_edges, const uint32_t* __restrict__ cost,
                                                          const uint32_t* __restrict__ magic, unsigned char* chain_mem,
                                                          size_t chain_stride, uint32_t n_snaps, uint32_t C,
                                                          const uint32_t* __restrict__ muts, uint32_t n_steps,
                                                          u64* __restrict__ out_ns, uint32_t* chain_flags, SearchDev search) {
    extern __shared__ __align__(16) unsigned char lds_raw[];
    const Tables T{ops, edges, in_edges, cost};
    // the chain's strategy is worked on in LDS (and written through to HBM), so that the many
    // uniform configuration look-ups do not queue behind the wavefront's stores to HBM
    uint2* cfg_lds = (uint2*)lds_raw;
    const WaveLds L = carve_lds(lds_raw + (size_t)S.n_ops_pad * 8, S);
    const uint32_t c = blockIdx.x;
    if (c >= C) return;
    const int lane = lane_id();
    const ChainMem cm = carve_chain(chain_mem + (size_t)c * chain_stride, S, n_snaps);
    const uint32_t magic_v = load_magic(magic);
    const uint32_t n_words = S.n_ops * WAVE;
    for (uint32_t i = lane; i < S.n_ops; i += WAVE) cfg_lds[i] = cm.cfgs[i];
    wave_sync();
    bool poisoned = first_u32(chain_flags[c]) != 0;
    ChainMeta meta = *cm.meta;
    meta.step = first_u64(meta.step);
    meta.n_valid = first_u32(meta.n_valid);
    meta.stale = first_u32(meta.stale);
    meta.n_steps = first_u64(meta.n_steps);
    meta.n_resumed = first_u64(meta.n_resumed);
    meta.n_events = first_u64(meta.n_events);
    meta.n_events_full = first_u64(meta.n_events_full);
    meta.cur_ns = first_u64(meta.cur_ns);
    meta.idle_steps = first_u64(meta.idle_steps);
    meta.n_converged = first_u64(meta.n_converged);
    meta.loc = first_u32(meta.loc);
    meta.tag = first_u32(meta.tag);
    Recorder rec{cm.end_try, cm.snap_words, cm.snap_l1, cm.snap_free, meta.step, 0, meta.loc, n_snaps, 1, 0, 0};
    Sim m{S, T, cfg_lds, cm.words, cm.exe_of, L, magic_v, 0, false, NO_OVERRIDE, make_uint2(0, 0), CACHE ? cm.ecache : nullptr, true};
    u64 best = search.enabled ? first_u64(search.best_ns[c]) : 0;
    if (search.enabled && !poisoned && !meta.stale && meta.cur_ns < best) {
        // the strategy the search starts from counts as seen
        best = meta.cur_ns;
        for (uint32_t i = lane; i < S.n_ops; i += WAVE) search.best_cfgs[(size_t)c * S.n_ops + i] = cfg_lds[i];
    }

    for (uint32_t s = 0; s < n_steps; s++) {
        Counters cnt = {};
        bool proposal = false, valid = true;
        uint32_t op = 0;
        uint2 ocfg = make_uint2(0, 0);
        if (search.enabled) {
            if (!poisoned && !meta.stale && !(search.patience && meta.idle_steps >= search.patience)) {
                const u64 st = search.first_step + s;
                op = first_u32((uint32_t)(draw64(search.seed, 10, c, st) % S.n_ops));
                const uint32_t t0 = first_u32(search.tuple_ptr[op]), t1 = first_u32(search.tuple_ptr[op + 1]);
                if (t1 > t0) {   // an op without a list gets no proposals
                    const uint32_t deg = search.tuples[t0 + (uint32_t)(draw64(search.seed, 11, c, st) % (t1 - t0))];
                    const uint32_t off = (uint32_t)(draw64(search.seed, 12, c, st) % S.n_dev);
                    ocfg = cfg_lds[op];
                    wave_sync();
                    if (lane == 0) cfg_lds[op] = make_uint2(first_u32(deg), first_u32(off) | (1u << 16));   // stride 1
                    wave_sync();
                    proposal = true;
                }
            }
        } else if (muts) {
            const uint32_t* mu = muts + ((size_t)s * C + c) * 3;
            op = first_u32(mu[0]);
            if (op >= S.n_ops) poisoned = true;
            if (!poisoned) {
                ocfg = cfg_lds[op];
                wave_sync();
                if (lane == 0) {
                    const uint2 ncfg = make_uint2(mu[1], mu[2]);
                    cfg_lds[op] = ncfg;
                    cm.cfgs[op] = ncfg;
                }
                wave_sync();
            }
        }
        u64 mk = RESULT_INVALID;
        StrategyClass cls = STRATEGY_INVALID;
        if (!poisoned) cls = validate_strategy(m);
        valid = cls != STRATEGY_INVALID;
        if (!poisoned && !valid && !proposal) { meta.stale = 1; meta.cur_ns = RESULT_INVALID; }
        const bool changed = muts != nullptr || proposal;
        if (changed && !poisoned) meta.n_steps++;
        bool accepted = false;

        if (search.enabled && !proposal && !poisoned && !meta.stale) {
            mk = meta.cur_ns;   // no proposal this step: nothing to simulate
        } else if (!poisoned && valid) {
            // where the simulation may start (0 = time 0)
            uint32_t k = 0, pend_new = 0;
            if (changed && !meta.stale && meta.n_valid > 1 && meta.step != 0) k = resume_point(m, cm.end_of, meta, op, ocfg, pend_new);
            const uint32_t capacity = n_snaps;
            // phase 1: makespan only, to fix the snapshot spacing (no snapshots yet);
            // phase 2: the recorded simulation
            int phase = (k == 0 && meta.step == 0) ? 1 : 2;
            u64 rc = 0;
            bool converged = false;
            while (phase < 3) {
                const bool record = phase == 2;
                const u64 before = cnt.n_events;
                if (record) {
                    meta.tag = meta.tag >= 0xffffu ? 0u : meta.tag;
                    if (meta.tag == 0) {
                        // tags start over: forget what earlier runs wrote
                        for (uint32_t t = lane; t < n_words; t += WAVE) cm.end_try[t] = 0;
                        __threadfence_block();
                        wave_sync();
                    }
                    meta.tag++;
                }
                rec.step = meta.step;
                rec.tag = (u64)meta.tag << 48;
                rec.loc = meta.loc;
                rec.n_snaps = record ? capacity : 0;
                rec.end_try = record ? cm.end_try : nullptr;
                rec.next = k + 1;
                // a resumed run of a changed strategy may re-join the accepted timeline
                rec.check_below = (record && k > 0 && changed) ? meta.n_valid : 0u;
                rec.check_op = op;
                if (k == 0) {
                    init_state(m, cnt);
                } else {
                    if (CACHE && record) refresh_ecache_for_op(m, op);
                    load_snapshot(m, rec, k);
                    // the loaded state still describes the op under its old configuration
                    patch_state_for_op(m, m.words, L.l1, op, ocfg, pend_new);
                    wave_sync();
                    rebuild_l2(m);
                }
                rc = cls == STRATEGY_REGULAR ? run_events<WIDE, true, true, false, TREE ? Q_TREE : Q_FLAT, CACHE>(m, cnt, rec)
                                             : run_events<WIDE, true, false, false, TREE ? Q_TREE : Q_FLAT, CACHE>(m, cnt, rec);
                if (rc == RUN_CONVERGED) { converged = true; rc = 0; mk = meta.cur_ns; break; }
                mk = rc ? rc : makespan(m);
                if (rc) break;
                if (phase == 1) { meta.step = (2 * mk) / capacity + 1; phase = 2; continue; }
                if (k == 0) meta.n_events_full = cnt.n_events - before;
                break;
            }
            if (changed) meta.n_events += cnt.n_events;
            // the decision: forced mutations and the starting strategy are always taken; a proposal
            // by the Metropolis rule (Section 6.1) with tabulated probabilities
            if (!rc) {
                accepted = true;
                if (proposal && mk > meta.cur_ns) {
                    u64 b = (mk - meta.cur_ns) / search.bucket_ns;
                    if (b >= search.n_buckets) b = search.n_buckets - 1;
                    const uint32_t u = (uint32_t)(draw64(search.seed, 13, c, search.first_step + s) >> 32);
                    accepted = u < search.accept[b];
                }
            }
            if (accepted) {
                if (proposal && lane == 0) cm.cfgs[op] = cfg_lds[op];
                if (k > 0) {
                    meta.n_resumed++;
                    // what the snapshots that stay hold about the op is rewritten for its new configuration
                    for (uint32_t sn = 1; sn <= k; sn++) {
                        const size_t at = (size_t)(((meta.loc >> sn) & 1u) * n_snaps + sn);
                        patch_state_for_op(m, cm.snap_words + at * n_words, cm.snap_l1 + at * S.n_ops_pad, op, ocfg, pend_new);
                    }
                }
                commit_run(cm, meta, rec, k + 1, n_words, converged);
                if (converged) meta.n_converged++;
                meta.stale = 0;
                meta.cur_ns = mk;
                // the spacing was fixed by an earlier makespan; if the timeline has become more than
                // twice shorter or longer, re-space: the snapshots are dropped and the next simulation
                // starts from time 0 with the new spacing
                const u64 ideal = (2 * mk) / capacity + 1;
                if (ideal * 2 < meta.step || ideal > meta.step * 2) { meta.step = ideal; meta.n_valid = 1; }
            } else if (proposal) {
                wave_sync();
                if (lane == 0) cfg_lds[op] = ocfg;
                wave_sync();
                if (CACHE) refresh_ecache_for_op(m, op);
                mk = meta.cur_ns;
            } else {
                // a forced step whose simulation failed (overflow): no timeline for this strategy
                meta.stale = 1;
                meta.n_valid = 0;
                meta.cur_ns = mk;
            }
        } else if (proposal && !valid) {
            // an invalid proposal is rejected
            wave_sync();
            if (lane == 0) cfg_lds[op] = ocfg;
            wave_sync();
            mk = meta.cur_ns;
        }
        if (search.enabled) meta.idle_steps++;
        if (search.enabled && !poisoned && mk < RESULT_OVERFLOW && mk < best) {
            best = mk;
            meta.idle_steps = 0;
            for (uint32_t i = lane; i < S.n_ops; i += WAVE) search.best_cfgs[(size_t)c * S.n_ops + i] = cfg_lds[i];
        }
        if (lane == 0) out_ns[(size_t)s * C + c] = mk;
        wave_sync();
    }
    if (lane == 0) {
        chain_flags[c] = poisoned ? 1u : 0u;
        *cm.meta = meta;
        if (search.enabled) search.best_ns[c] = best;
    }
}

// Trial mutations (the proposals of Section 6.2 before acceptance): evaluates M alternative
// single-op mutations per chain, each against the chain's current strategy and stored
// timeline, without changing the chain.  One wavefront per (proposal, chain); its task words
// live in a private workspace slot, the chain's snapshots are only read.
template <bool WIDE, bool TREE, bool CACHE>
__global__ __launch_bounds__(WAVE) void k_sim_chain_try(SimDev S, const DOp* __restrict__ ops, const DEdge* __restrict__ edges,
                                                        const DEdge* __restrict__ in_edges, const uint32_t* __restrict__ cost,
                                                        const uint32_t* __restrict__ magic, const unsigned char* __restrict__ chain_mem,
                                                        size_t chain_stride, uint32_t n_snaps, uint32_t C,
                                                        const uint32_t* __restrict__ muts, uint32_t M, u64* __restrict__ out_ns,
                                                        const uint32_t* __restrict__ chain_flags, uint32_t* __restrict__ next_item,
                                                        unsigned char* __restrict__ ws, size_t slot_stride) {
    extern __shared__ __align__(16) unsigned char lds_raw[];
    const Tables T{ops, edges, in_edges, cost};
    const WaveLds L = carve_lds(lds_raw, S);
    const uint32_t magic_v = load_magic(magic);
    unsigned char* slot = ws + (size_t)blockIdx.x * slot_stride;
    u64* words = (u64*)slot;
    uint32_t* exe_of = (uint32_t*)(slot + (size_t)S.n_ops * WAVE * 8);
    const uint32_t total = M * C;
    // proposals differ a lot in cost (how much of the timeline they keep): wavefronts draw the
    // next one from a counter instead of striding
    for (;;) {
        uint32_t id = 0;
        if (lane_id() == 0) id = atomicAdd(next_item, 1u);
        id = first_u32(id);
        if (id >= total) break;
        const uint32_t c = id % C;
        // the chain is only read here
        const ChainMem cm = carve_chain(const_cast<unsigned char*>(chain_mem) + (size_t)c * chain_stride, S, n_snaps);
        ChainMeta meta = *cm.meta;
        meta.step = first_u64(meta.step);
        meta.n_valid = first_u32(meta.n_valid);
        meta.stale = first_u32(meta.stale);
        const uint32_t* mu = muts + (size_t)id * 3;     // [M][C] records {op, cfg.x, cfg.y}
        const uint32_t op = first_u32(mu[0]);
        u64 mk = RESULT_INVALID;
        if (op < S.n_ops && first_u32(chain_flags[c]) == 0) {
            const uint2 ocfg = cm.cfgs[op];
            SimTrial m{S, T, cm.cfgs, words, exe_of, L, magic_v, 0, false, op, make_uint2(first_u32(mu[1]), first_u32(mu[2])),
                       CACHE ? cm.ecache : nullptr, false};
            const StrategyClass cls = validate_strategy(m);
            if (cls != STRATEGY_INVALID) {
                Counters cnt = {};
                Recorder rec{nullptr, cm.snap_words, cm.snap_l1, cm.snap_free, meta.step, 0, first_u32(meta.loc), n_snaps, 1, 0, 0};
                uint32_t k = 0, pend_new = 0;
                if (!meta.stale && meta.n_valid > 1 && meta.step != 0) k = resume_point(m, cm.end_of, meta, op, ocfg, pend_new);
                if (k == 0) {
                    init_state(m, cnt);
                } else {
                    load_snapshot(m, rec, k);
                    patch_state_for_op(m, m.words, L.l1, op, ocfg, pend_new);
                    wave_sync();
                    rebuild_l2(m);
                }
                const u64 rc = cls == STRATEGY_REGULAR ? run_events<WIDE, false, true, false, TREE ? Q_TREE : Q_FLAT, CACHE>(m, cnt, rec) : run_events<WIDE, false, false, false, TREE ? Q_TREE : Q_FLAT, CACHE>(m, cnt, rec);
                mk = rc ? rc : makespan(m);
            }
        }
        if (lane_id() == 0) out_ns[id] = mk;
        wave_sync();
    }
}

// clears the work counter of k_sim_chain_try (a kernel, so that a captured stream sees a node)
// ---- neighbour sweep (Section 8: is a strategy locally optimal?) --------------------------
//
// The neighbours of a strategy differ from it in the configuration of one op.  Neighbour k of
// the enumeration: ops op_begin..op_end-1 in order; per op every degree tuple of its list, in
// list order; per tuple every device offset 0..n_dev-1; stride 1.  first[o - op_begin] is the
// index of the first neighbour of op o.  Writes the same mutation for every chain ([M][C]).
__global__ __launch_bounds__(WAVE) void k_neighbour_list(const uint32_t* __restrict__ tuple_ptr, const uint32_t* __restrict__ tuples,
                                                         const uint32_t* __restrict__ first, uint32_t op_begin, uint32_t op_end,
                                                         uint32_t n_dev, uint32_t M, uint32_t C, uint32_t* __restrict__ muts) {
    const uint32_t k = blockIdx.x * WAVE + threadIdx.x;
    if (k >= M) return;
    // binary search for the op whose range holds k
    uint32_t lo = 0, hi = op_end - op_begin;       // first[lo] <= k < first[hi]
    while (hi - lo > 1) {
        const uint32_t mid = (lo + hi) / 2;
        if (first[mid] <= k) lo = mid; else hi = mid;
    }
    const uint32_t op = op_begin + lo;
    const uint32_t r = k - first[lo];
    const uint32_t deg = tuples[tuple_ptr[op] + r / n_dev];
    const uint32_t off = r % n_dev;
    for (uint32_t c = 0; c < C; c++) {
        uint32_t* mu = muts + ((size_t)k * C + c) * 3;
        mu[0] = op; mu[1] = deg; mu[2] = off | (1u << 16);
    }
}

// per chain: the smallest time among its M results ([M][C]) and the lowest index that has it;
// one wavefront per chain
__global__ __launch_bounds__(WAVE) void k_best_of(const u64* __restrict__ ns, uint32_t M, uint32_t C, u64* __restrict__ best_ns,
                                                  uint32_t* __restrict__ best_idx) {
    const uint32_t c = blockIdx.x;
    if (c >= C) return;
    u64 b = ~0ull;
    uint32_t bi = 0xffffffffu;
    for (uint32_t k = lane_id(); k < M; k += WAVE) {
        const u64 v = ns[(size_t)k * C + c];
        if (v < b) { b = v; bi = k; }        // ascending k: the first index wins inside a lane
    }
    const u64 m = wave_min_u64(b);
    const uint32_t mi = wave_min_u32(b == m ? bi : 0xffffffffu);
    if (lane_id() == 0) { best_ns[c] = m; best_idx[c] = mi; }
}

__global__ void k_zero_u32(uint32_t* p) { if (threadIdx.x == 0 && blockIdx.x == 0) *p = 0; }

}  // namespace ffsim
